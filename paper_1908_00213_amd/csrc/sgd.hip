// chn_sgd_update / chn_sgd_update_multi: param <- param - lr * grad (Section "Background and
// Motivation" names stochastic gradient descent as the optimiser of the run phase), optionally
// refreshing a bfloat16 working copy of a mixed-precision master weight in the same pass.
// HBM-bound: 12 bytes per parameter (14 with the working copy), 16-byte accesses.  The multi-tensor
// form updates a whole parameter set with one launch: the tensor table travels in the kernel
// arguments and every block finds its tensor by a short scan of the per-tensor block prefix.
#include "common.h"

namespace chn {
namespace {

constexpr int kThreads = 256;
constexpr int kVecPerThread = 4;                       // 4 x float4 per thread
constexpr int kElemsPerBlock = kThreads * kVecPerThread * 4;
constexpr int kMaxTensors = 40;

__device__ __forceinline__ void sgd_block(float *p, const float *g, bf16_raw *lp, int64_t n, int64_t block, float lr, bool vec) {
  const int64_t base = block * kElemsPerBlock;
  if (vec) {
    float4 pv[kVecPerThread], gv[kVecPerThread];
#pragma unroll
    for (int u = 0; u < kVecPerThread; ++u) {
      const int64_t e = base + ((int64_t)u * kThreads + threadIdx.x) * 4;
      if (e + 3 < n) { pv[u] = *reinterpret_cast<const float4 *>(p + e); gv[u] = *reinterpret_cast<const float4 *>(g + e); }
    }
#pragma unroll
    for (int u = 0; u < kVecPerThread; ++u) {
      const int64_t e = base + ((int64_t)u * kThreads + threadIdx.x) * 4;
      if (e + 3 < n) {
        float4 r;
        r.x = pv[u].x - lr * gv[u].x; r.y = pv[u].y - lr * gv[u].y;
        r.z = pv[u].z - lr * gv[u].z; r.w = pv[u].w - lr * gv[u].w;
        *reinterpret_cast<float4 *>(p + e) = r;
        if (lp) {
          uint2 w;
          w.x = (uint32_t)f32_to_bf16(r.x) | ((uint32_t)f32_to_bf16(r.y) << 16);
          w.y = (uint32_t)f32_to_bf16(r.z) | ((uint32_t)f32_to_bf16(r.w) << 16);
          *reinterpret_cast<uint2 *>(lp + e) = w;
        }
      } else {
        for (int64_t i = e; i < n && i < e + 4; ++i) {
          const float r = p[i] - lr * g[i];
          p[i] = r;
          if (lp) lp[i] = f32_to_bf16(r);
        }
      }
    }
  } else {
    for (int u = 0; u < kVecPerThread * 4; ++u) {
      const int64_t i = base + (int64_t)u * kThreads + threadIdx.x;
      if (i < n) {
        const float r = p[i] - lr * g[i];
        p[i] = r;
        if (lp) lp[i] = f32_to_bf16(r);
      }
    }
  }
}

struct MultiArgs {
  float *p[kMaxTensors];
  const float *g[kMaxTensors];
  bf16_raw *lp[kMaxTensors];
  int64_t n[kMaxTensors];
  int block_end[kMaxTensors];   // exclusive prefix end of each tensor's blocks
  int vec[kMaxTensors];
  int count;
  float lr;
};

__global__ __launch_bounds__(kThreads) void sgd_multi_kernel(MultiArgs a) {
  int t = 0;
  while (t + 1 < a.count && (int)blockIdx.x >= a.block_end[t]) ++t;
  const int first = t == 0 ? 0 : a.block_end[t - 1];
  sgd_block(a.p[t], a.g[t], a.lp[t], a.n[t], (int64_t)blockIdx.x - first, a.lr, a.vec[t] != 0);
}

chn_status check_triple(const chn_array *param, const chn_array *grad, const chn_array *lowp, int64_t *n, bool *vec) {
  CHN_TRY(validate(param, "param", true));
  CHN_TRY(validate(grad, "grad", false));
  if (param->dtype != CHN_F32 || grad->dtype != CHN_F32) return fail(CHN_ERR_DTYPE, "sgd: param and grad must be F32");
  if (param->ndim != grad->ndim) return fail(CHN_ERR_SHAPE, "sgd: param and grad shapes differ");
  for (int d = 0; d < param->ndim; ++d)
    if (param->shape[d] != grad->shape[d]) return fail(CHN_ERR_SHAPE, "sgd: param and grad shapes differ");
  if (!is_contiguous(param) || !is_contiguous(grad)) return fail(CHN_ERR_STRIDE, "sgd: param and grad must be contiguous");
  *n = numel(param);
  *vec = reinterpret_cast<uintptr_t>(param->data) % 16 == 0 && reinterpret_cast<uintptr_t>(grad->data) % 16 == 0;
  if (lowp) {
    CHN_TRY(validate(lowp, "lowp_copy", true));
    if (lowp->dtype != CHN_BF16) return fail(CHN_ERR_DTYPE, "sgd: lowp_copy must be BF16");
    if (numel(lowp) != *n || lowp->ndim != param->ndim) return fail(CHN_ERR_SHAPE, "sgd: lowp_copy shape differs from param");
    for (int d = 0; d < param->ndim; ++d)
      if (param->shape[d] != lowp->shape[d]) return fail(CHN_ERR_SHAPE, "sgd: lowp_copy shape differs from param");
    if (!is_contiguous(lowp)) return fail(CHN_ERR_STRIDE, "sgd: lowp_copy must be contiguous");
    *vec = *vec && reinterpret_cast<uintptr_t>(lowp->data) % 8 == 0;
  }
  return CHN_OK;
}

}  // namespace
}  // namespace chn

extern "C" {

chn_status chn_sgd_update_multi(int n, const chn_array *const *params, const chn_array *const *grads,
                                float lr, const chn_array *const *lowp_copies, chn_stream stream) {
  using namespace chn;
  if (n < 0) return fail(CHN_ERR_SHAPE, "sgd: negative tensor count");
  if (n == 0) return CHN_OK;
  if (!params || !grads) return fail(CHN_ERR_NULL, "sgd: tensor list is NULL");
  // validate everything before the first launch so that a failing call enqueues nothing
  for (int i = 0; i < n; ++i) {
    int64_t cnt; bool vec;
    CHN_TRY(check_triple(params[i], grads[i], lowp_copies ? lowp_copies[i] : nullptr, &cnt, &vec));
    if ((cnt + kElemsPerBlock - 1) / kElemsPerBlock > 0x3fffffff) return fail(CHN_ERR_SHAPE, "sgd: tensor too large");
  }
  int i = 0;
  while (i < n) {
    MultiArgs a{};
    a.lr = lr;
    int64_t blocks = 0;
    while (i < n && a.count < kMaxTensors) {
      int64_t cnt; bool vec;
      check_triple(params[i], grads[i], lowp_copies ? lowp_copies[i] : nullptr, &cnt, &vec);
      const int64_t nb = (cnt + kElemsPerBlock - 1) / kElemsPerBlock;
      if (cnt > 0) {
        if (blocks + nb > 0x7fffffff) break;
        const int k = a.count++;
        a.p[k] = static_cast<float *>(params[i]->data);
        a.g[k] = static_cast<const float *>(grads[i]->data);
        a.lp[k] = (lowp_copies && lowp_copies[i]) ? static_cast<bf16_raw *>(lowp_copies[i]->data) : nullptr;
        a.n[k] = cnt;
        a.vec[k] = vec ? 1 : 0;
        blocks += nb;
        a.block_end[k] = (int)blocks;
      }
      ++i;
    }
    if (a.count == 0) continue;
    hipLaunchKernelGGL(sgd_multi_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, as_stream(stream), a);
    CHN_TRY(check_launch("sgd_update"));
  }
  return CHN_OK;
}

chn_status chn_sgd_update(const chn_array *param, const chn_array *grad, float lr,
                          const chn_array *lowp_copy, chn_stream stream) {
  const chn_array *p[1] = {param}, *g[1] = {grad}, *l[1] = {lowp_copy};
  return chn_sgd_update_multi(1, p, g, lr, l, stream);
}

}  // extern "C"
