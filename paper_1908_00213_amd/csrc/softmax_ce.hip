// chn_softmax_ce_fwd / chn_softmax_ce_bwd: row-wise softmax cross-entropy (textbook definition; the
// paper only names the classification task, Section "API Design").
//
// A group of G lanes (8 / 64 / 256 by row length) owns one row.  The forward pass reads the row once
// with 16-byte loads, keeping a running (max, sum of exp) pair per lane that is merged through wave
// butterflies (and LDS for G = 256); a second one-block kernel folds the per-row losses into the mean
// in a fixed order.  The backward pass reads the row (twice when the log-sum-exp was not retained:
// the second read comes from L2) and writes the gradient once.  HBM-bound for wide rows.
#include "common.h"

namespace chn {
namespace {

struct MS { float m, s; };  // running max and sum of exp(x - m)

__device__ __forceinline__ MS ms_merge(MS a, MS b) {
  const float m = fmaxf(a.m, b.m);
  if (m == -INFINITY) return MS{m, 0.0f};
  return MS{m, a.s * expf(a.m - m) + b.s * expf(b.m - m)};
}

template <int G>
__device__ __forceinline__ MS group_merge(MS v, MS *smem /* [4] per block, G==256 only */) {
  constexpr int W = G < 64 ? G : 64;
#pragma unroll
  for (int o = W / 2; o > 0; o >>= 1) {
    MS other{__shfl_xor(v.m, o, 64), __shfl_xor(v.s, o, 64)};
    v = ms_merge(v, other);
  }
  if constexpr (G == 256) {
    if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = v;
    __syncthreads();
    v = ms_merge(ms_merge(smem[0], smem[1]), ms_merge(smem[2], smem[3]));
    __syncthreads();
  }
  return v;
}

// Running (max, sum exp) of one row slice owned by lane g of G.
template <typename T, int G, bool VEC>
__device__ __forceinline__ MS row_scan(const T *p, int64_t C, int g) {
  MS acc{-INFINITY, 0.0f};
  if constexpr (VEC) {
    constexpr int N = Vec16<T>::N;
    const int64_t nvec = C / N;
    // Four vectors per round: their loads are in flight together, the running sum is rescaled once
    // per round, and the exponentials are the hardware's (exp2 of a pre-scaled argument; the arguments
    // are <= 0 and the relative error of a term is a few 1e-7, far inside what the log of the sum
    // needs).  With the library's expf this loop was bound by arithmetic, not by memory.
    int64_t v = g;
    for (; v + 3 * G < nvec; v += 4 * G) {
      Vec16<T> x[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) x[u].load(p + (v + u * G) * N);
      float mx = x[0].get(0);
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int i = 0; i < N; ++i) mx = fmaxf(mx, x[u].get(i));
      const float m = fmaxf(acc.m, mx);
      float s = acc.s * __expf(acc.m - m);
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int i = 0; i < N; ++i) s += __expf(x[u].get(i) - m);
      acc = MS{m, s};
    }
    for (; v < nvec; v += G) {
      Vec16<T> x;
      x.load(p + v * N);
      float mx = x.get(0);
#pragma unroll
      for (int i = 1; i < N; ++i) mx = fmaxf(mx, x.get(i));
      const float m = fmaxf(acc.m, mx);
      float s = acc.s * __expf(acc.m - m);
#pragma unroll
      for (int i = 0; i < N; ++i) s += __expf(x.get(i) - m);
      acc = MS{m, s};
    }
    for (int64_t c = nvec * N + g; c < C; c += G) {
      const float x = Elem<T>::load(p + c);
      const float m = fmaxf(acc.m, x);
      acc = MS{m, acc.s * expf(acc.m - m) + expf(x - m)};
    }
  } else {
    for (int64_t c = g; c < C; c += G) {
      const float x = Elem<T>::load(p + c);
      const float m = fmaxf(acc.m, x);
      acc = MS{m, acc.s * expf(acc.m - m) + expf(x - m)};
    }
  }
  return acc;
}

// The label of a row as the kernels use it: a value outside [0, C) is never used as an offset -- such a
// row is treated like one that carries `ignore` (no loss, no gradient, not counted among the valid rows).
template <typename L>
__device__ __forceinline__ int64_t row_label(const L *labels, int64_t row, int64_t ignore, int64_t C) {
  const int64_t t = (int64_t)labels[row];
  return (uint64_t)t < (uint64_t)C ? t : ignore;
}

template <typename T, typename L, int G, bool VEC>
__global__ __launch_bounds__(256) void sce_fwd_kernel(const T *z, int64_t pitch, const L *labels, int64_t N, int64_t C,
                                                      int64_t ignore, float *loss_rows, float *lse_out) {
  __shared__ MS smem[4];
  const int g = threadIdx.x % G;
  int64_t row = (int64_t)blockIdx.x * (256 / G) + threadIdx.x / G;
  const bool live = row < N;
  if (!live) row = N - 1;  // keep every lane in the collectives; results are discarded
  const T *p = z + row * pitch;
  MS v = group_merge<G>(row_scan<T, G, VEC>(p, C, g), smem);
  if (g == 0 && live) {
    const float lse = v.m + logf(v.s);
    const int64_t t = row_label(labels, row, ignore, C);
    if (lse_out) lse_out[row] = lse;
    loss_rows[row] = t == ignore ? 0.0f : lse - Elem<T>::load(p + t);
  }
}

// loss_mean = sum of loss_rows over valid rows / number of valid rows, fixed order.
template <typename L>
__global__ __launch_bounds__(1024) void sce_mean_kernel(const float *loss_rows, const L *labels, int64_t N, int64_t C, int64_t ignore,
                                                        float *loss_mean) {
  __shared__ float ssum[16];
  __shared__ int scnt[16];
  float s = 0.0f;
  int cnt = 0;
  for (int64_t n = threadIdx.x; n < N; n += 1024)
    if (row_label(labels, n, ignore, C) != ignore) { s += loss_rows[n]; ++cnt; }
  s = wave_sum(s);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, 64);
  if ((threadIdx.x & 63) == 0) { ssum[threadIdx.x >> 6] = s; scnt[threadIdx.x >> 6] = cnt; }
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = 0.0f;
    int c = 0;
    for (int w = 0; w < 16; ++w) { t += ssum[w]; c += scnt[w]; }
    *loss_mean = c > 0 ? t / (float)c : 0.0f;
  }
}

// scale = upstream / N_valid (0 when no row is valid)
template <typename L>
__global__ __launch_bounds__(1024) void sce_scale_kernel(const L *labels, int64_t N, int64_t C, int64_t ignore, float upstream, float *scale) {
  __shared__ int scnt[16];
  int cnt = 0;
  for (int64_t n = threadIdx.x; n < N; n += 1024) cnt += (row_label(labels, n, ignore, C) != ignore) ? 1 : 0;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, 64);
  if ((threadIdx.x & 63) == 0) scnt[threadIdx.x >> 6] = cnt;
  __syncthreads();
  if (threadIdx.x == 0) {
    int c = 0;
    for (int w = 0; w < 16; ++w) c += scnt[w];
    *scale = c > 0 ? upstream / (float)c : 0.0f;
  }
}

// Gradient of one row, lane g of G: dz[c] = scale * (exp(z[c] - lse) - [c == t]).
template <typename T, typename TO, int G, bool VEC>
__device__ __forceinline__ void row_grad(const T *p, TO *q, int64_t C, int g, int64_t t, float lse, float scale) {
  if constexpr (VEC) {
    constexpr int NI = Vec16<T>::N, NO = Vec16<TO>::N;
    constexpr int E = NI > NO ? NI : NO;  // elements per step: whole 16-byte vectors on both sides
    const int64_t nstep = C / E;
    for (int64_t v = g; v < nstep; v += G) {
      Vec16<T> x[E / NI];
      Vec16<TO> y[E / NO];
#pragma unroll
      for (int i = 0; i < E / NI; ++i) x[i].load(p + v * E + i * NI);
#pragma unroll
      for (int i = 0; i < E; ++i) {
        const int64_t c = v * E + i;
        float pr = scale == 0.0f ? 0.0f : expf(x[i / NI].get(i % NI) - lse);
        y[i / NO].set(i % NO, scale * (pr - (c == t ? 1.0f : 0.0f)));
      }
#pragma unroll
      for (int i = 0; i < E / NO; ++i) y[i].store(q + v * E + i * NO);
    }
    for (int64_t c = nstep * E + g; c < C; c += G) {
      float pr = scale == 0.0f ? 0.0f : expf(Elem<T>::load(p + c) - lse);
      Elem<TO>::store(q + c, scale * (pr - (c == t ? 1.0f : 0.0f)));
    }
  } else {
    for (int64_t c = g; c < C; c += G) {
      float pr = scale == 0.0f ? 0.0f : expf(Elem<T>::load(p + c) - lse);
      Elem<TO>::store(q + c, scale * (pr - (c == t ? 1.0f : 0.0f)));
    }
  }
}

template <typename T, typename TO, typename L, int G, bool VEC>
__global__ __launch_bounds__(256) void sce_bwd_kernel(const T *z, int64_t pitch, const L *labels, int64_t N, int64_t C,
                                                      int64_t ignore, const float *lse_in, const float *scale_ptr,
                                                      TO *dz, int64_t dpitch) {
  __shared__ MS smem[4];
  const int g = threadIdx.x % G;
  int64_t row = (int64_t)blockIdx.x * (256 / G) + threadIdx.x / G;
  const bool live = row < N;
  if (!live) row = N - 1;
  const T *p = z + row * pitch;
  float lse;
  if (lse_in) {
    lse = lse_in[row];
  } else {
    MS v = group_merge<G>(row_scan<T, G, VEC>(p, C, g), smem);
    lse = v.m + logf(v.s);
  }
  if (!live) return;
  const int64_t t = row_label(labels, row, ignore, C);
  const float scale = t == ignore ? 0.0f : *scale_ptr;
  row_grad<T, TO, G, VEC>(p, dz + row * dpitch, C, g, t, lse, scale);
}

// Forward and backward of a row in one visit: log-sum-exp and loss first, then the gradient while the
// row is still in the caches (the logits travel from HBM once instead of twice).  dz may be the
// logits' own buffer: a lane overwrites only elements that it has read itself, after the whole row
// has been scanned.
template <typename T, typename TO, typename L, int G, bool VEC>
__global__ __launch_bounds__(256) void sce_fused_kernel(const T *z, int64_t pitch, const L *labels, int64_t N, int64_t C,
                                                        int64_t ignore, const float *scale_ptr, float *loss_rows, float *lse_out,
                                                        TO *dz, int64_t dpitch) {
  __shared__ MS smem[4];
  const int g = threadIdx.x % G;
  int64_t row = (int64_t)blockIdx.x * (256 / G) + threadIdx.x / G;
  const bool live = row < N;
  if (!live) row = N - 1;
  const T *p = z + row * pitch;
  const MS v = group_merge<G>(row_scan<T, G, VEC>(p, C, g), smem);
  const float lse = v.m + logf(v.s);
  const int64_t t = row_label(labels, row, ignore, C);
  float zt = 0.0f;
  if (g == 0 && live && t != ignore) zt = Elem<T>::load(p + t);   // (read before the row may be overwritten)
  if constexpr (G == 256) __syncthreads();
  else __builtin_amdgcn_wave_barrier();
  if (!live) return;
  if (g == 0) {
    if (lse_out) lse_out[row] = lse;
    loss_rows[row] = t == ignore ? 0.0f : lse - zt;
  }
  row_grad<T, TO, G, VEC>(p, dz + row * dpitch, C, g, t, lse, t == ignore ? 0.0f : *scale_ptr);
}

// The same with the row held in registers between the scan and the gradient: a lane keeps its SMAX steps of E
// elements (whole 16-byte vectors on both sides), so the logits are read exactly once, also where the rows that
// the chip has in flight do not fit its L2s (4480 x 10000 fp32: 86 -> 60 us).  Needs C % E == 0 and C / E <= SMAX * G.
template <typename T, typename TO, typename L, int G, int SMAX>
__global__ __launch_bounds__(256) void sce_fused_reg_kernel(const T *z, int64_t pitch, const L *labels, int64_t N, int64_t C,
                                                            int64_t ignore, const float *scale_ptr, float *loss_rows, float *lse_out,
                                                            TO *dz, int64_t dpitch) {
  constexpr int NI = Vec16<T>::N, NO = Vec16<TO>::N, E = NI > NO ? NI : NO;
  __shared__ MS smem[4];
  const int g = threadIdx.x % G;
  int64_t row = (int64_t)blockIdx.x * (256 / G) + threadIdx.x / G;
  const bool live = row < N;
  if (!live) row = N - 1;
  const T *p = z + row * pitch;
  const int64_t nstep = C / E;
  float x[SMAX][E];
  float m = -INFINITY;
#pragma unroll
  for (int u = 0; u < SMAX; ++u) {
    const int64_t v = g + (int64_t)u * G;
    if (v < nstep) {
      Vec16<T> in[E / NI];
#pragma unroll
      for (int i = 0; i < E / NI; ++i) in[i].load(p + v * E + i * NI);
#pragma unroll
      for (int i = 0; i < E; ++i) { x[u][i] = in[i / NI].get(i % NI); m = fmaxf(m, x[u][i]); }
    } else {
#pragma unroll
      for (int i = 0; i < E; ++i) x[u][i] = -INFINITY;
    }
  }
  float sum = 0.0f;
  if (g < nstep) {                                     // (a lane without elements contributes (-inf, 0))
#pragma unroll
    for (int u = 0; u < SMAX; ++u)
#pragma unroll
      for (int i = 0; i < E; ++i) sum += __expf(x[u][i] - m);
  }
  const MS v = group_merge<G>(MS{m, sum}, smem);
  const float lse = v.m + logf(v.s);
  const int64_t t = row_label(labels, row, ignore, C);
  float zt = 0.0f;
  if (g == 0 && live && t != ignore) zt = Elem<T>::load(p + t);   // (read before the row may be overwritten)
  if constexpr (G == 256) __syncthreads();
  else __builtin_amdgcn_wave_barrier();
  if (!live) return;
  if (g == 0) {
    if (lse_out) lse_out[row] = lse;
    loss_rows[row] = t == ignore ? 0.0f : lse - zt;
  }
  const float scale = t == ignore ? 0.0f : *scale_ptr;
  TO *q = dz + row * dpitch;
#pragma unroll
  for (int u = 0; u < SMAX; ++u) {
    const int64_t vs = g + (int64_t)u * G;
    if (vs < nstep) {
      Vec16<TO> y[E / NO];
#pragma unroll
      for (int i = 0; i < E; ++i) {
        const int64_t c = vs * E + i;
        const float pr = scale == 0.0f ? 0.0f : expf(x[u][i] - lse);
        y[i / NO].set(i % NO, scale * (pr - (c == t ? 1.0f : 0.0f)));
      }
#pragma unroll
      for (int i = 0; i < E / NO; ++i) y[i].store(q + vs * E + i * NO);
    }
  }
}

// A whole small problem (few classes, a few thousand rows) in one launch of one block: count the
// valid rows, then every thread takes rows tid, tid + 1024, ... from log-sum-exp to gradient, then the
// mean loss in a fixed order.  For the small MLP steps, which are bound by the number of launches.
// A row (at most CR classes) is held in registers: its loads are all in flight at once and it is read
// from memory once.
template <typename T, typename TO, typename L, int CR>
__global__ __launch_bounds__(1024) void sce_small_kernel(const T *z, int64_t pitch, const L *labels, int64_t N, int64_t C,
                                                         int64_t ignore, float upstream, float *loss_mean, float *lse_out,
                                                         TO *dz, int64_t dpitch) {
  __shared__ float ssum[16];
  __shared__ int scnt[16];
  int cnt = 0;
  for (int64_t n = threadIdx.x; n < N; n += 1024) cnt += (row_label(labels, n, ignore, C) != ignore) ? 1 : 0;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, 64);
  if ((threadIdx.x & 63) == 0) scnt[threadIdx.x >> 6] = cnt;
  __syncthreads();
  int valid = 0;
  for (int w = 0; w < 16; ++w) valid += scnt[w];
  const float scale_all = valid > 0 ? upstream / (float)valid : 0.0f;
  float s = 0.0f;
  for (int64_t n = threadIdx.x; n < N; n += 1024) {
    const T *p = z + n * pitch;
    const int64_t t = row_label(labels, n, ignore, C);
    float x[CR];
#pragma unroll
    for (int c = 0; c < CR; ++c) x[c] = c < C ? Elem<T>::load(p + c) : -INFINITY;   // exp(-inf - m) = 0
    float m = -INFINITY;
#pragma unroll
    for (int c = 0; c < CR; ++c) m = fmaxf(m, x[c]);
    float e = 0.0f, xt = 0.0f;
#pragma unroll
    for (int c = 0; c < CR; ++c) {
      if (c < C) e += expf(x[c] - m);
      xt = c == t ? x[c] : xt;
    }
    const float lse = m + logf(e);
    if (lse_out) lse_out[n] = lse;
    if (t != ignore) s += lse - xt;
    const float scale = t == ignore ? 0.0f : scale_all;
    TO *q = dz + n * dpitch;
#pragma unroll
    for (int c = 0; c < CR; ++c) {
      if (c < C) {
        const float pr = scale == 0.0f ? 0.0f : expf(x[c] - lse);
        Elem<TO>::store(q + c, scale * (pr - (c == t ? 1.0f : 0.0f)));
      }
    }
  }
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) ssum[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    float tot = 0.0f;
    for (int w = 0; w < 16; ++w) tot += ssum[w];
    *loss_mean = valid > 0 ? tot / (float)valid : 0.0f;
  }
}

// The derivative of the gradient (what differentiating a backward pass needs): with
// G[n,c] = s_n (p[n,c] - [c == t_n]), s_n = upstream / N_valid on valid rows and 0 elsewhere, and u the
// gradient that reaches G,
//   dz[n,c]   = s_n p[n,c] (u[n,c] - sum_k p[n,k] u[n,k])        (G's dependence on the logits)
//   rows[n]   = sum_c u[n,c] (p[n,c] - [c == t_n])                (summed over valid rows / N_valid: d upstream)
// One wave per row, three sweeps (log-sum-exp unless given, the two row sums, the result): this path is
// taken by second-order derivatives only.  F32 throughout.
template <typename L>
__global__ __launch_bounds__(256) void sce_bwd2_kernel(const float *z, int64_t pitch, const L *labels, int64_t N, int64_t C, int64_t ignore,
                                                       const float *lse_in, const float *scale_ptr, const float *u, int64_t upitch,
                                                       float *dz, int64_t dpitch, float *rows) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= N) return;
  const float *p = z + row * pitch, *ur = u + row * upitch;
  float lse;
  if (lse_in) {
    lse = lse_in[row];
  } else {
    float m = -INFINITY;
    for (int64_t c = lane; c < C; c += 64) m = fmaxf(m, p[c]);
    m = wave_max(m);
    float e = 0.0f;
    for (int64_t c = lane; c < C; c += 64) e += expf(p[c] - m);
    lse = m + logf(wave_sum(e));
  }
  const int64_t t = row_label(labels, row, ignore, C);
  float pu = 0.0f;
  for (int64_t c = lane; c < C; c += 64) pu += expf(p[c] - lse) * ur[c];
  pu = wave_sum(pu);
  const bool valid = t != ignore;
  if (rows && lane == 0) rows[row] = valid ? pu - ur[t] : 0.0f;
  const float s = valid ? *scale_ptr : 0.0f;
  float *q = dz + row * dpitch;
  for (int64_t c = lane; c < C; c += 64) q[c] = s == 0.0f ? 0.0f : s * expf(p[c] - lse) * (ur[c] - pu);
}

struct Common {
  int64_t N = 0, C = 0, pitch = 0;
  int G = 256;
  bool vec = false;
};

chn_status check_common(const chn_array *logits, const chn_array *labels, Common *c) {
  CHN_TRY(validate(logits, "logits", false));
  CHN_TRY(validate(labels, "labels", false));
  if (!is_float(logits->dtype)) return fail(CHN_ERR_DTYPE, "softmax_ce: logits must be F32 or BF16");
  if (!is_index(labels->dtype)) return fail(CHN_ERR_DTYPE, "softmax_ce: labels must be I32 or I64");
  CHN_TRY(row_major_2d(logits, "logits", &c->N, &c->C, &c->pitch));
  if (labels->ndim != 1 || labels->shape[0] != c->N)
    return fail(CHN_ERR_SHAPE, "softmax_ce: labels must have shape (%lld,)", (long long)c->N);
  if (!is_contiguous(labels)) return fail(CHN_ERR_STRIDE, "softmax_ce: labels must be contiguous");
  if (c->N > 0 && c->C == 0) return fail(CHN_ERR_SHAPE, "softmax_ce: zero classes");
  c->G = c->C >= 2048 ? 256 : (c->C > 32 ? 64 : 8);
  const int n = 16 / dtype_size(logits->dtype);
  c->vec = reinterpret_cast<uintptr_t>(logits->data) % 16 == 0 && c->pitch % n == 0;
  return CHN_OK;
}

chn_status check_rows_f32(const chn_array *a, const char *name, int64_t N) {
  CHN_TRY(validate(a, name, true));
  if (a->dtype != CHN_F32) return fail(CHN_ERR_DTYPE, "softmax_ce: %s must be F32", name);
  if (a->ndim != 1 || a->shape[0] != N) return fail(CHN_ERR_SHAPE, "softmax_ce: %s must have shape (%lld,)", name, (long long)N);
  if (!is_contiguous(a)) return fail(CHN_ERR_STRIDE, "softmax_ce: %s must be contiguous", name);
  return CHN_OK;
}

inline size_t round256(size_t n) { return (n + 255) / 256 * 256; }

template <typename T, typename L>
void launch_fwd(const Common &c, const chn_array *logits, const chn_array *labels, int64_t ignore, float *rows, float *lse, hipStream_t st) {
  const T *z = static_cast<const T *>(logits->data);
  const L *t = static_cast<const L *>(labels->data);
#define CHN_FWD(G, V) hipLaunchKernelGGL((sce_fwd_kernel<T, L, G, V>), dim3((unsigned)((c.N + 256 / G - 1) / (256 / G))), dim3(256), 0, st, z, c.pitch, t, c.N, c.C, ignore, rows, lse)
  if (c.G == 256) { if (c.vec) CHN_FWD(256, true); else CHN_FWD(256, false); }
  else if (c.G == 64) { if (c.vec) CHN_FWD(64, true); else CHN_FWD(64, false); }
  else CHN_FWD(8, false);
#undef CHN_FWD
}

template <typename T, typename TO, typename L>
void launch_bwd(const Common &c, const chn_array *logits, const chn_array *labels, int64_t ignore, const float *lse,
                const float *scale, const chn_array *dl, int64_t dpitch, bool vec, hipStream_t st) {
  const T *z = static_cast<const T *>(logits->data);
  const L *t = static_cast<const L *>(labels->data);
  TO *d = static_cast<TO *>(dl->data);
#define CHN_BWD(G, V) hipLaunchKernelGGL((sce_bwd_kernel<T, TO, L, G, V>), dim3((unsigned)((c.N + 256 / G - 1) / (256 / G))), dim3(256), 0, st, z, c.pitch, t, c.N, c.C, ignore, lse, scale, d, dpitch)
  if (c.G == 256) { if (vec) CHN_BWD(256, true); else CHN_BWD(256, false); }
  else if (c.G == 64) { if (vec) CHN_BWD(64, true); else CHN_BWD(64, false); }
  else CHN_BWD(8, false);
#undef CHN_BWD
}

template <typename T, typename TO, typename L>
void launch_fused(const Common &c, const chn_array *logits, const chn_array *labels, int64_t ignore, const float *scale, float *rows,
                  float *lse, const chn_array *dl, int64_t dpitch, bool vec, hipStream_t st) {
  const T *z = static_cast<const T *>(logits->data);
  const L *t = static_cast<const L *>(labels->data);
  TO *d = static_cast<TO *>(dl->data);
  // long rows that fit a block's registers (48 elements per lane: up to 12288 classes) are read once
  constexpr int kE = (16 / (int)sizeof(T)) > (16 / (int)sizeof(TO)) ? (16 / (int)sizeof(T)) : (16 / (int)sizeof(TO));
  constexpr int kSteps = 48 / kE;
  if (vec && c.C % kE == 0 && c.G == 256 && c.C / kE <= (int64_t)kSteps * 256) {
    hipLaunchKernelGGL((sce_fused_reg_kernel<T, TO, L, 256, kSteps>), dim3((unsigned)c.N), dim3(256), 0, st, z, c.pitch, t, c.N, c.C, ignore, scale, rows, lse, d, dpitch);
    return;
  }
#define CHN_FUSED(G, V) hipLaunchKernelGGL((sce_fused_kernel<T, TO, L, G, V>), dim3((unsigned)((c.N + 256 / G - 1) / (256 / G))), dim3(256), 0, st, z, c.pitch, t, c.N, c.C, ignore, scale, rows, lse, d, dpitch)
  if (c.G == 256) { if (vec) CHN_FUSED(256, true); else CHN_FUSED(256, false); }
  else if (c.G == 64) { if (vec) CHN_FUSED(64, true); else CHN_FUSED(64, false); }
  else CHN_FUSED(8, false);
#undef CHN_FUSED
}

template <typename T, typename TO, typename L>
void launch_small(const Common &c, const chn_array *logits, const chn_array *labels, int64_t ignore, float upstream, float *loss_mean,
                  float *lse, const chn_array *dl, int64_t dpitch, hipStream_t st) {
  if (c.C <= 16)
    hipLaunchKernelGGL((sce_small_kernel<T, TO, L, 16>), dim3(1), dim3(1024), 0, st, static_cast<const T *>(logits->data), c.pitch,
                       static_cast<const L *>(labels->data), c.N, c.C, ignore, upstream, loss_mean, lse, static_cast<TO *>(dl->data), dpitch);
  else
    hipLaunchKernelGGL((sce_small_kernel<T, TO, L, 64>), dim3(1), dim3(1024), 0, st, static_cast<const T *>(logits->data), c.pitch,
                       static_cast<const L *>(labels->data), c.N, c.C, ignore, upstream, loss_mean, lse, static_cast<TO *>(dl->data), dpitch);
}

}  // namespace
}  // namespace chn

extern "C" {

size_t chn_softmax_ce_workspace_bytes(int64_t n_rows) {
  if (n_rows < 0) n_rows = 0;
  return 256 + chn::round256((size_t)n_rows * sizeof(float));
}

chn_status chn_softmax_ce_fwd(const chn_array *logits, const chn_array *labels, int64_t ignore_label,
                              const chn_array *loss_mean, const chn_array *loss_rows,
                              const chn_array *lse, void *ws, size_t ws_bytes, chn_stream stream) {
  using namespace chn;
  Common c;
  CHN_TRY(check_common(logits, labels, &c));
  CHN_TRY(validate(loss_mean, "loss_mean", true));
  if (loss_mean->dtype != CHN_F32 || numel(loss_mean) != 1)
    return fail(CHN_ERR_SHAPE, "softmax_ce: loss_mean must be a single F32 value");
  if (loss_rows) CHN_TRY(check_rows_f32(loss_rows, "loss_rows", c.N));
  if (lse) CHN_TRY(check_rows_f32(lse, "lse", c.N));
  float *rows = loss_rows ? static_cast<float *>(loss_rows->data) : nullptr;
  if (!rows && c.N > 0) {
    CHN_TRY(check_ws(ws, ws_bytes, chn_softmax_ce_workspace_bytes(c.N), "softmax_ce_fwd"));
    rows = reinterpret_cast<float *>(static_cast<char *>(ws) + 256);
  }
  hipStream_t st = as_stream(stream);
  if (c.N > 0) {
    float *l = lse ? static_cast<float *>(lse->data) : nullptr;
    const bool i32 = labels->dtype == CHN_I32;
    if (logits->dtype == CHN_F32) {
      if (i32) launch_fwd<float, int32_t>(c, logits, labels, ignore_label, rows, l, st);
      else launch_fwd<float, int64_t>(c, logits, labels, ignore_label, rows, l, st);
    } else {
      if (i32) launch_fwd<bf16_raw, int32_t>(c, logits, labels, ignore_label, rows, l, st);
      else launch_fwd<bf16_raw, int64_t>(c, logits, labels, ignore_label, rows, l, st);
    }
    CHN_TRY(check_launch("softmax_ce_fwd rows"));
  }
  float *lm = static_cast<float *>(loss_mean->data);
  if (labels->dtype == CHN_I32)
    hipLaunchKernelGGL((sce_mean_kernel<int32_t>), dim3(1), dim3(1024), 0, st, rows, static_cast<const int32_t *>(labels->data), c.N, c.C, ignore_label, lm);
  else
    hipLaunchKernelGGL((sce_mean_kernel<int64_t>), dim3(1), dim3(1024), 0, st, rows, static_cast<const int64_t *>(labels->data), c.N, c.C, ignore_label, lm);
  return check_launch("softmax_ce_fwd mean");
}

chn_status chn_softmax_ce_bwd(const chn_array *logits, const chn_array *labels, int64_t ignore_label,
                              const chn_array *lse, float upstream, const chn_array *dlogits,
                              void *ws, size_t ws_bytes, chn_stream stream) {
  using namespace chn;
  Common c;
  CHN_TRY(check_common(logits, labels, &c));
  CHN_TRY(validate(dlogits, "dlogits", true));
  if (!is_float(dlogits->dtype)) return fail(CHN_ERR_DTYPE, "softmax_ce: dlogits must be F32 or BF16");
  int64_t dn, dc, dpitch;
  CHN_TRY(row_major_2d(dlogits, "dlogits", &dn, &dc, &dpitch));
  if (dn != c.N || dc != c.C) return fail(CHN_ERR_SHAPE, "softmax_ce: dlogits must have the logits' shape");
  if (lse) CHN_TRY(check_rows_f32(lse, "lse", c.N));
  if (c.N == 0) return CHN_OK;
  CHN_TRY(check_ws(ws, ws_bytes, 256, "softmax_ce_bwd"));
  float *scale = static_cast<float *>(ws);
  hipStream_t st = as_stream(stream);
  const bool i32 = labels->dtype == CHN_I32;
  if (i32) hipLaunchKernelGGL((sce_scale_kernel<int32_t>), dim3(1), dim3(1024), 0, st, static_cast<const int32_t *>(labels->data), c.N, c.C, ignore_label, upstream, scale);
  else hipLaunchKernelGGL((sce_scale_kernel<int64_t>), dim3(1), dim3(1024), 0, st, static_cast<const int64_t *>(labels->data), c.N, c.C, ignore_label, upstream, scale);
  CHN_TRY(check_launch("softmax_ce_bwd scale"));
  const int no = 16 / dtype_size(dlogits->dtype);
  const bool vec = c.vec && reinterpret_cast<uintptr_t>(dlogits->data) % 16 == 0 && dpitch % no == 0;
  const float *l = lse ? static_cast<const float *>(lse->data) : nullptr;
  const bool zin32 = logits->dtype == CHN_F32, zout32 = dlogits->dtype == CHN_F32;
#define CHN_GO(T, TO)                                                                                        \
  do {                                                                                                       \
    if (i32) launch_bwd<T, TO, int32_t>(c, logits, labels, ignore_label, l, scale, dlogits, dpitch, vec, st); \
    else launch_bwd<T, TO, int64_t>(c, logits, labels, ignore_label, l, scale, dlogits, dpitch, vec, st);     \
  } while (0)
  if (zin32 && zout32) CHN_GO(float, float);
  else if (zin32 && !zout32) CHN_GO(float, bf16_raw);
  else if (!zin32 && zout32) CHN_GO(bf16_raw, float);
  else CHN_GO(bf16_raw, bf16_raw);
#undef CHN_GO
  return check_launch("softmax_ce_bwd rows");
}

chn_status chn_softmax_ce_bwd2(const chn_array *logits, const chn_array *labels, int64_t ignore_label,
                               const chn_array *lse, float upstream, const chn_array *gg, const chn_array *dlogits,
                               const chn_array *dupstream, void *ws, size_t ws_bytes, chn_stream stream) {
  using namespace chn;
  Common c;
  CHN_TRY(check_common(logits, labels, &c));
  CHN_TRY(validate(gg, "gg", false));
  CHN_TRY(validate(dlogits, "dlogits", true));
  if (logits->dtype != CHN_F32 || gg->dtype != CHN_F32 || dlogits->dtype != CHN_F32)
    return fail(CHN_ERR_DTYPE, "softmax_ce_bwd2: logits, gg and dlogits must be F32");
  int64_t un, uc, upitch, dn, dc, dpitch;
  CHN_TRY(row_major_2d(gg, "gg", &un, &uc, &upitch));
  CHN_TRY(row_major_2d(dlogits, "dlogits", &dn, &dc, &dpitch));
  if (un != c.N || uc != c.C || dn != c.N || dc != c.C) return fail(CHN_ERR_SHAPE, "softmax_ce_bwd2: gg and dlogits must have the logits' shape");
  if (lse) CHN_TRY(check_rows_f32(lse, "lse", c.N));
  if (dupstream) {
    CHN_TRY(validate(dupstream, "dupstream", true));
    if (dupstream->dtype != CHN_F32 || numel(dupstream) != 1) return fail(CHN_ERR_SHAPE, "softmax_ce_bwd2: dupstream must be a single F32 value");
  }
  if (c.N == 0) return CHN_OK;
  CHN_TRY(check_ws(ws, ws_bytes, chn_softmax_ce_workspace_bytes(c.N), "softmax_ce_bwd2"));
  float *scale = static_cast<float *>(ws);
  float *rows = dupstream ? reinterpret_cast<float *>(static_cast<char *>(ws) + 256) : nullptr;
  hipStream_t st = as_stream(stream);
  const float *l = lse ? static_cast<const float *>(lse->data) : nullptr;
  const unsigned blocks = (unsigned)((c.N + 3) / 4);
#define CHN_GO(L)                                                                                                              \
  do {                                                                                                                         \
    const L *t = static_cast<const L *>(labels->data);                                                                         \
    hipLaunchKernelGGL((sce_scale_kernel<L>), dim3(1), dim3(1024), 0, st, t, c.N, c.C, ignore_label, upstream, scale);          \
    hipLaunchKernelGGL((sce_bwd2_kernel<L>), dim3(blocks), dim3(256), 0, st, static_cast<const float *>(logits->data), c.pitch, t, \
                       c.N, c.C, ignore_label, l, scale, static_cast<const float *>(gg->data), upitch,                          \
                       static_cast<float *>(dlogits->data), dpitch, rows);                                                     \
    if (dupstream) hipLaunchKernelGGL((sce_mean_kernel<L>), dim3(1), dim3(1024), 0, st, rows, t, c.N, c.C, ignore_label,        \
                                      static_cast<float *>(dupstream->data));                                                  \
  } while (0)
  if (labels->dtype == CHN_I32) CHN_GO(int32_t); else CHN_GO(int64_t);
#undef CHN_GO
  return check_launch("softmax_ce_bwd2");
}

chn_status chn_softmax_ce_fwd_bwd(const chn_array *logits, const chn_array *labels, int64_t ignore_label,
                                  const chn_array *loss_mean, const chn_array *lse, float upstream,
                                  const chn_array *dlogits, void *ws, size_t ws_bytes, chn_stream stream) {
  using namespace chn;
  Common c;
  CHN_TRY(check_common(logits, labels, &c));
  CHN_TRY(validate(loss_mean, "loss_mean", true));
  if (loss_mean->dtype != CHN_F32 || numel(loss_mean) != 1)
    return fail(CHN_ERR_SHAPE, "softmax_ce: loss_mean must be a single F32 value");
  if (lse) CHN_TRY(check_rows_f32(lse, "lse", c.N));
  CHN_TRY(validate(dlogits, "dlogits", true));
  if (!is_float(dlogits->dtype)) return fail(CHN_ERR_DTYPE, "softmax_ce: dlogits must be F32 or BF16");
  int64_t dn, dc, dpitch;
  CHN_TRY(row_major_2d(dlogits, "dlogits", &dn, &dc, &dpitch));
  if (dn != c.N || dc != c.C) return fail(CHN_ERR_SHAPE, "softmax_ce: dlogits must have the logits' shape");
  if (c.N > 0 && dlogits->data == logits->data && (dlogits->dtype != logits->dtype || dpitch != c.pitch))
    return fail(CHN_ERR_STRIDE, "softmax_ce: a gradient written over the logits needs their dtype and row pitch");
  hipStream_t st = as_stream(stream);
  float *lm = static_cast<float *>(loss_mean->data);
  float *l = lse ? static_cast<float *>(lse->data) : nullptr;
  const bool i32 = labels->dtype == CHN_I32;
  const bool zin32 = logits->dtype == CHN_F32, zout32 = dlogits->dtype == CHN_F32;
  if (c.N == 0 || (c.C <= 64 && c.N <= 8192)) {         // (no rows: the mean of nothing is written as 0)
#define CHN_GO(T, TO)                                                                                        \
  do {                                                                                                       \
    if (i32) launch_small<T, TO, int32_t>(c, logits, labels, ignore_label, upstream, lm, l, dlogits, dpitch, st); \
    else launch_small<T, TO, int64_t>(c, logits, labels, ignore_label, upstream, lm, l, dlogits, dpitch, st);     \
  } while (0)
    if (zin32 && zout32) CHN_GO(float, float);
    else if (zin32 && !zout32) CHN_GO(float, bf16_raw);
    else if (!zin32 && zout32) CHN_GO(bf16_raw, float);
    else CHN_GO(bf16_raw, bf16_raw);
#undef CHN_GO
    return check_launch("softmax_ce_fwd_bwd (one block)");
  }
  CHN_TRY(check_ws(ws, ws_bytes, chn_softmax_ce_workspace_bytes(c.N), "softmax_ce_fwd_bwd"));
  float *scale = static_cast<float *>(ws);
  float *rows = reinterpret_cast<float *>(static_cast<char *>(ws) + 256);
  if (i32) hipLaunchKernelGGL((sce_scale_kernel<int32_t>), dim3(1), dim3(1024), 0, st, static_cast<const int32_t *>(labels->data), c.N, c.C, ignore_label, upstream, scale);
  else hipLaunchKernelGGL((sce_scale_kernel<int64_t>), dim3(1), dim3(1024), 0, st, static_cast<const int64_t *>(labels->data), c.N, c.C, ignore_label, upstream, scale);
  CHN_TRY(check_launch("softmax_ce_fwd_bwd scale"));
  const int no = 16 / dtype_size(dlogits->dtype);
  const bool vec = c.vec && reinterpret_cast<uintptr_t>(dlogits->data) % 16 == 0 && dpitch % no == 0;
#define CHN_GO(T, TO)                                                                                              \
  do {                                                                                                             \
    if (i32) launch_fused<T, TO, int32_t>(c, logits, labels, ignore_label, scale, rows, l, dlogits, dpitch, vec, st); \
    else launch_fused<T, TO, int64_t>(c, logits, labels, ignore_label, scale, rows, l, dlogits, dpitch, vec, st);     \
  } while (0)
  if (zin32 && zout32) CHN_GO(float, float);
  else if (zin32 && !zout32) CHN_GO(float, bf16_raw);
  else if (!zin32 && zout32) CHN_GO(bf16_raw, float);
  else CHN_GO(bf16_raw, bf16_raw);
#undef CHN_GO
  CHN_TRY(check_launch("softmax_ce_fwd_bwd rows"));
  if (i32) hipLaunchKernelGGL((sce_mean_kernel<int32_t>), dim3(1), dim3(1024), 0, st, rows, static_cast<const int32_t *>(labels->data), c.N, c.C, ignore_label, lm);
  else hipLaunchKernelGGL((sce_mean_kernel<int64_t>), dim3(1), dim3(1024), 0, st, rows, static_cast<const int64_t *>(labels->data), c.N, c.C, ignore_label, lm);
  return check_launch("softmax_ce_fwd_bwd mean");
}

}  // extern "C"
