// chn_adam_update_multi: the Adam optimiser (the paper names it as an optimiser choice in the code
// figure of Section "Distributed Parallel Training"; the update itself is Algorithm 1 of Kingma & Ba,
// "Adam: A Method for Stochastic Optimization"):
//   m <- b1 m + (1 - b1) g          v <- b2 v + (1 - b2) g^2
//   p <- p - lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps)
// for a whole parameter set in as few launches as the kernel argument space allows; optionally
// refreshes the bfloat16 working copy of a mixed-precision master weight in the same pass.
// HBM-bound: 28 bytes per parameter (16 read, 12 written; 30 with the working copy), 16-byte accesses.
#include <cmath>

#include "common.h"

namespace chn {
namespace {

constexpr int kThreads = 256;
constexpr int kVecPerThread = 2;                       // 2 x float4 per thread and array
constexpr int kElemsPerBlock = kThreads * kVecPerThread * 4;
constexpr int kMaxTensors = 24;

struct AdamCoef { float b1, b2, one_minus_b1, one_minus_b2, inv_c1, inv_c2, lr, eps; };

__device__ __forceinline__ float adam_one(float p, float g, float &m, float &v, const AdamCoef &k) {
  m = k.b1 * m + k.one_minus_b1 * g;
  v = k.b2 * v + k.one_minus_b2 * g * g;
  return p - k.lr * (m * k.inv_c1) / (sqrtf(v * k.inv_c2) + k.eps);
}

struct AdamArgs {
  float *p[kMaxTensors];
  const float *g[kMaxTensors];
  float *m[kMaxTensors];
  float *v[kMaxTensors];
  bf16_raw *lp[kMaxTensors];
  int64_t n[kMaxTensors];
  int block_end[kMaxTensors];   // exclusive prefix end of each tensor's blocks
  int vec[kMaxTensors];
  int count;
  AdamCoef k;
};

__global__ __launch_bounds__(kThreads) void adam_multi_kernel(AdamArgs a) {
  int t = 0;
  while (t + 1 < a.count && (int)blockIdx.x >= a.block_end[t]) ++t;
  const int64_t block = (int64_t)blockIdx.x - (t == 0 ? 0 : a.block_end[t - 1]);
  float *p = a.p[t], *m = a.m[t], *v = a.v[t];
  const float *g = a.g[t];
  bf16_raw *lp = a.lp[t];
  const int64_t n = a.n[t], base = block * kElemsPerBlock;
  if (a.vec[t]) {
    float4 pv[kVecPerThread], gv[kVecPerThread], mv[kVecPerThread], vv[kVecPerThread];
#pragma unroll
    for (int u = 0; u < kVecPerThread; ++u) {
      const int64_t e = base + ((int64_t)u * kThreads + threadIdx.x) * 4;
      if (e + 3 < n) {
        pv[u] = *reinterpret_cast<const float4 *>(p + e); gv[u] = *reinterpret_cast<const float4 *>(g + e);
        mv[u] = *reinterpret_cast<const float4 *>(m + e); vv[u] = *reinterpret_cast<const float4 *>(v + e);
      }
    }
#pragma unroll
    for (int u = 0; u < kVecPerThread; ++u) {
      const int64_t e = base + ((int64_t)u * kThreads + threadIdx.x) * 4;
      if (e + 3 < n) {
        float4 r;
        r.x = adam_one(pv[u].x, gv[u].x, mv[u].x, vv[u].x, a.k); r.y = adam_one(pv[u].y, gv[u].y, mv[u].y, vv[u].y, a.k);
        r.z = adam_one(pv[u].z, gv[u].z, mv[u].z, vv[u].z, a.k); r.w = adam_one(pv[u].w, gv[u].w, mv[u].w, vv[u].w, a.k);
        *reinterpret_cast<float4 *>(p + e) = r;
        *reinterpret_cast<float4 *>(m + e) = mv[u];
        *reinterpret_cast<float4 *>(v + e) = vv[u];
        if (lp) {
          uint2 w;
          w.x = (uint32_t)f32_to_bf16(r.x) | ((uint32_t)f32_to_bf16(r.y) << 16);
          w.y = (uint32_t)f32_to_bf16(r.z) | ((uint32_t)f32_to_bf16(r.w) << 16);
          *reinterpret_cast<uint2 *>(lp + e) = w;
        }
      } else {
        for (int64_t i = e; i < n && i < e + 4; ++i) {
          float mi = m[i], vi = v[i];
          const float r = adam_one(p[i], g[i], mi, vi, a.k);
          p[i] = r; m[i] = mi; v[i] = vi;
          if (lp) lp[i] = f32_to_bf16(r);
        }
      }
    }
  } else {
    for (int u = 0; u < kVecPerThread * 4; ++u) {
      const int64_t i = base + (int64_t)u * kThreads + threadIdx.x;
      if (i < n) {
        float mi = m[i], vi = v[i];
        const float r = adam_one(p[i], g[i], mi, vi, a.k);
        p[i] = r; m[i] = mi; v[i] = vi;
        if (lp) lp[i] = f32_to_bf16(r);
      }
    }
  }
}

chn_status same_f32(const chn_array *a, const char *name, const chn_array *ref, bool out, bool *vec) {
  CHN_TRY(validate(a, name, out));
  if (a->dtype != CHN_F32) return fail(CHN_ERR_DTYPE, "adam: %s must be F32", name);
  if (a->ndim != ref->ndim) return fail(CHN_ERR_SHAPE, "adam: %s differs in shape from param", name);
  for (int d = 0; d < ref->ndim; ++d)
    if (a->shape[d] != ref->shape[d]) return fail(CHN_ERR_SHAPE, "adam: %s differs in shape from param", name);
  if (!is_contiguous(a)) return fail(CHN_ERR_STRIDE, "adam: %s must be contiguous", name);
  *vec = *vec && reinterpret_cast<uintptr_t>(a->data) % 16 == 0;
  return CHN_OK;
}

chn_status check_set(const chn_array *p, const chn_array *g, const chn_array *m, const chn_array *v, const chn_array *lowp,
                     int64_t *n, bool *vec) {
  if (!p) return fail(CHN_ERR_NULL, "adam: param is NULL");
  *vec = true;
  CHN_TRY(same_f32(p, "param", p, true, vec));
  if (!g || !m || !v) return fail(CHN_ERR_NULL, "adam: grad, m or v is NULL");
  CHN_TRY(same_f32(g, "grad", p, false, vec));
  CHN_TRY(same_f32(m, "m", p, true, vec));
  CHN_TRY(same_f32(v, "v", p, true, vec));
  *n = numel(p);
  if (lowp) {
    CHN_TRY(validate(lowp, "lowp_copy", true));
    if (lowp->dtype != CHN_BF16) return fail(CHN_ERR_DTYPE, "adam: lowp_copy must be BF16");
    if (lowp->ndim != p->ndim) return fail(CHN_ERR_SHAPE, "adam: lowp_copy differs in shape from param");
    for (int d = 0; d < p->ndim; ++d)
      if (lowp->shape[d] != p->shape[d]) return fail(CHN_ERR_SHAPE, "adam: lowp_copy differs in shape from param");
    if (!is_contiguous(lowp)) return fail(CHN_ERR_STRIDE, "adam: lowp_copy must be contiguous");
    *vec = *vec && reinterpret_cast<uintptr_t>(lowp->data) % 8 == 0;
  }
  return CHN_OK;
}

}  // namespace
}  // namespace chn

extern "C" chn_status chn_adam_update_multi(int n, const chn_array *const *params, const chn_array *const *grads,
                                            const chn_array *const *ms, const chn_array *const *vs, double lr, double beta1,
                                            double beta2, double eps, int64_t step, const chn_array *const *lowp_copies,
                                            chn_stream stream) {
  using namespace chn;
  if (n < 0) return fail(CHN_ERR_SHAPE, "adam: negative tensor count");
  if (step < 1) return fail(CHN_ERR_OP, "adam: step counts from 1, got %lld", (long long)step);
  if (!(beta1 >= 0.0 && beta1 < 1.0 && beta2 >= 0.0 && beta2 < 1.0)) return fail(CHN_ERR_OP, "adam: beta1 and beta2 must lie in [0, 1)");
  if (n == 0) return CHN_OK;
  if (!params || !grads || !ms || !vs) return fail(CHN_ERR_NULL, "adam: tensor list is NULL");
  for (int i = 0; i < n; ++i) {
    int64_t cnt; bool vec;
    CHN_TRY(check_set(params[i], grads[i], ms[i], vs[i], lowp_copies ? lowp_copies[i] : nullptr, &cnt, &vec));
    if ((cnt + kElemsPerBlock - 1) / kElemsPerBlock > 0x3fffffff) return fail(CHN_ERR_SHAPE, "adam: tensor too large");
  }
  AdamCoef k;
  // every coefficient is formed in double precision and rounded to fp32 once
  k.b1 = (float)beta1; k.b2 = (float)beta2; k.one_minus_b1 = (float)(1.0 - beta1); k.one_minus_b2 = (float)(1.0 - beta2);
  k.inv_c1 = (float)(1.0 / (1.0 - std::pow(beta1, (double)step)));
  k.inv_c2 = (float)(1.0 / (1.0 - std::pow(beta2, (double)step)));
  k.lr = (float)lr; k.eps = (float)eps;
  int i = 0;
  while (i < n) {
    AdamArgs a{};
    a.k = k;
    int64_t blocks = 0;
    while (i < n && a.count < kMaxTensors) {
      int64_t cnt; bool vec;
      check_set(params[i], grads[i], ms[i], vs[i], lowp_copies ? lowp_copies[i] : nullptr, &cnt, &vec);
      const int64_t nb = (cnt + kElemsPerBlock - 1) / kElemsPerBlock;
      if (cnt > 0) {
        if (blocks + nb > 0x7fffffff) break;
        const int j = a.count++;
        a.p[j] = static_cast<float *>(params[i]->data);
        a.g[j] = static_cast<const float *>(grads[i]->data);
        a.m[j] = static_cast<float *>(ms[i]->data);
        a.v[j] = static_cast<float *>(vs[i]->data);
        a.lp[j] = (lowp_copies && lowp_copies[i]) ? static_cast<bf16_raw *>(lowp_copies[i]->data) : nullptr;
        a.n[j] = cnt;
        a.vec[j] = vec ? 1 : 0;
        blocks += nb;
        a.block_end[j] = (int)blocks;
      }
      ++i;
    }
    if (a.count == 0) continue;
    hipLaunchKernelGGL(adam_multi_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, as_stream(stream), a);
    CHN_TRY(check_launch("adam_update"));
  }
  return CHN_OK;
}
