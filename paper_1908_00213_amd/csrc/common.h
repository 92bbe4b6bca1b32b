// Internal helpers shared by the libchn translation units (host validation + device utilities).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstdarg>
#include <cstdio>

#include "chn.h"

namespace chn {

// ---- error reporting -------------------------------------------------------------------------
char *last_error_buffer();  // thread-local, 512 bytes

inline chn_status fail(chn_status code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(last_error_buffer(), 512, fmt, ap);
  va_end(ap);
  return code;
}

#define CHN_TRY(expr)                        \
  do {                                       \
    chn_status _st = (expr);                 \
    if (_st != CHN_OK) return _st;           \
  } while (0)

inline chn_status check_launch(const char *what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(CHN_ERR_LAUNCH, "%s: %s", what, hipGetErrorString(e));
  return CHN_OK;
}

// ---- descriptor helpers ------------------------------------------------------------------------
inline int dtype_size(int dt) {
  switch (dt) {
    case CHN_F32: return 4;
    case CHN_BF16: return 2;
    case CHN_I32: return 4;
    case CHN_I64: return 8;
  }
  return 0;
}

inline bool is_float(int dt) { return dt == CHN_F32 || dt == CHN_BF16; }
inline bool is_index(int dt) { return dt == CHN_I32 || dt == CHN_I64; }

inline int64_t numel(const chn_array *a) {
  int64_t n = 1;
  for (int d = 0; d < a->ndim; ++d) n *= a->shape[d];
  return n;
}

// Checks pointer, ndim, dtype, shape >= 0, strides >= 0 and multiples of the item size.
// `is_output` additionally refuses zero strides on dimensions longer than 1.
chn_status validate(const chn_array *a, const char *name, bool is_output);

// True when the view is C-contiguous (dimensions of size 1 may carry any stride).
bool is_contiguous(const chn_array *a);

// Requires a 2-d view with unit stride along the last axis; returns the row pitch in elements.
chn_status row_major_2d(const chn_array *a, const char *name, int64_t *rows, int64_t *cols,
                        int64_t *pitch);

inline hipStream_t as_stream(chn_stream s) { return reinterpret_cast<hipStream_t>(s); }

inline chn_status check_ws(const void *ws, size_t have, size_t need, const char *what) {
  if (need == 0) return CHN_OK;
  if (!ws) return fail(CHN_ERR_WORKSPACE, "%s: workspace of %zu bytes required, got NULL", what, need);
  if (reinterpret_cast<uintptr_t>(ws) % 256)
    return fail(CHN_ERR_WORKSPACE, "%s: workspace must be 256-byte aligned", what);
  if (have < need)
    return fail(CHN_ERR_WORKSPACE, "%s: workspace of %zu bytes required, got %zu", what, need, have);
  return CHN_OK;
}

// ---- device-side scalar helpers ----------------------------------------------------------------
#if defined(__HIPCC__)
typedef uint16_t bf16_raw;

__device__ __forceinline__ float bf16_to_f32(bf16_raw b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// Round to nearest, ties to even (NaN stays NaN).
__device__ __forceinline__ bf16_raw f32_to_bf16(float f) {
  __bf16 h = static_cast<__bf16>(f);
  return __builtin_bit_cast(bf16_raw, h);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float *p) { return *p; }
  static __device__ __forceinline__ void store(float *p, float v) { *p = v; }
};
template <> struct Elem<bf16_raw> {
  static __device__ __forceinline__ float load(const bf16_raw *p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(bf16_raw *p, float v) { *p = f32_to_bf16(v); }
};

typedef float chn_f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t chn_u32x4 __attribute__((ext_vector_type(4)));

// 16-byte vector of T, converted to/from fp32 lanes.  The *_nt forms carry the non-temporal hint:
// streamed data that is touched once should not displace what the caches hold.
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  float4 raw;
  __device__ __forceinline__ void load(const float *p) { raw = *reinterpret_cast<const float4 *>(p); }
  __device__ __forceinline__ void store(float *p) const { *reinterpret_cast<float4 *>(p) = raw; }
  __device__ __forceinline__ void load_nt(const float *p) {
    const chn_f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const chn_f32x4 *>(p));
    raw = make_float4(v[0], v[1], v[2], v[3]);
  }
  __device__ __forceinline__ void store_nt(float *p) const {
    const chn_f32x4 v = {raw.x, raw.y, raw.z, raw.w};
    __builtin_nontemporal_store(v, reinterpret_cast<chn_f32x4 *>(p));
  }
  __device__ __forceinline__ float get(int i) const { return (&raw.x)[i]; }
  __device__ __forceinline__ void set(int i, float v) { (&raw.x)[i] = v; }
};
template <> struct Vec16<bf16_raw> {
  static constexpr int N = 8;
  uint4 raw;
  __device__ __forceinline__ void load(const bf16_raw *p) { raw = *reinterpret_cast<const uint4 *>(p); }
  __device__ __forceinline__ void store(bf16_raw *p) const { *reinterpret_cast<uint4 *>(p) = raw; }
  __device__ __forceinline__ void load_nt(const bf16_raw *p) {
    const chn_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const chn_u32x4 *>(p));
    raw = make_uint4(v[0], v[1], v[2], v[3]);
  }
  __device__ __forceinline__ void store_nt(bf16_raw *p) const {
    const chn_u32x4 v = {raw.x, raw.y, raw.z, raw.w};
    __builtin_nontemporal_store(v, reinterpret_cast<chn_u32x4 *>(p));
  }
  __device__ __forceinline__ float get(int i) const {
    uint32_t w = (&raw.x)[i >> 1];
    return __uint_as_float((i & 1) ? (w & 0xffff0000u) : (w << 16));
  }
  __device__ __forceinline__ void set(int i, float v) {
    uint32_t b = f32_to_bf16(v);
    uint32_t &w = (&raw.x)[i >> 1];
    w = (i & 1) ? ((w & 0x0000ffffu) | (b << 16)) : ((w & 0xffff0000u) | b);
  }
};

// erfc with a relative error of about 1e-6 everywhere, tails included: the Chebyshev fit
// erfc(z) ~ t exp(-z^2 + P(t)), t = 1 / (1 + z/2), z >= 0, of Numerical Recipes' "erfcc" (fractional
// error below 1.2e-7 in exact arithmetic; the fp32 evaluation of the exponent adds up to a few 1e-6
// for large z), reflected for negative arguments.  One reciprocal, one exponential, nine fused
// multiply-adds: a quarter of the library's erfcf, which made the element-wise gelu kernels
// arithmetic-bound.
__device__ __forceinline__ float erfc_f(float y) {
  const float z = fabsf(y);
  const float t = __builtin_amdgcn_rcpf(fmaf(0.5f, z, 1.0f));
  float p = fmaf(t, 0.17087277f, -0.82215223f);
  p = fmaf(t, p, 1.48851587f);
  p = fmaf(t, p, -1.13520398f);
  p = fmaf(t, p, 0.27886807f);
  p = fmaf(t, p, -0.18628806f);
  p = fmaf(t, p, 0.09678418f);
  p = fmaf(t, p, 0.37409196f);
  p = fmaf(t, p, 1.00002368f);
  p = fmaf(t, p, -1.26551223f);
  const float r = t * __expf(fmaf(-z, z, p));
  return y >= 0.0f ? r : 2.0f - r;
}
// gelu(x) = x * Phi(x); Phi written with erfc so that the negative tail keeps its relative accuracy.
__device__ __forceinline__ float gelu_f(float x) {
  return 0.5f * x * erfc_f(-x * 0.70710678118654752440f);
}
__device__ __forceinline__ float gelu_grad_f(float x) {
  float Phi = 0.5f * erfc_f(-x * 0.70710678118654752440f);
  float phi = 0.39894228040143267794f * __expf(-0.5f * x * x);
  return Phi + x * phi;
}
// Compact forms for GEMM epilogues, where the argument already carries the rounding error of a long
// fp32 sum and the code is replicated for every accumulator a lane holds.  Phi(x) comes from the
// classical five-term rational approximation of erf (Abramowitz & Stegun 7.1.26, absolute error
// below 1.5e-7), whose exp(-x^2/2) factor is shared with the density phi(x); for x < 0 the form
// 0.5 * poly * exp(-x^2/2) involves no cancellation.  One hardware exp and one hardware reciprocal.
// Written so that few instructions depend on each other and none is spent on what algebra removes:
// constants are folded into the arguments of the reciprocal and the exponential and into the
// polynomial, and gelu(x) = x * Phi(x) = max(x, 0) - |x| * Phi(-|x|) needs no case distinction.
struct PhiParts { float tail, e; };   // tail = Phi(-|x|), e = exp(-x^2 / 2)
__device__ __forceinline__ PhiParts phi_parts(float x) {
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f * 0.70710678118654752440f, fabsf(x), 1.0f));
  const float e = __builtin_amdgcn_exp2f(x * x * -0.72134752044448170368f);   // -log2(e) / 2
  const float poly = t * fmaf(t, fmaf(t, fmaf(t, fmaf(t, 0.5f * 1.061405429f, 0.5f * -1.453152027f), 0.5f * 1.421413741f),
                                      0.5f * -0.284496736f), 0.5f * 0.254829592f);
  return PhiParts{poly * e, e};
}
// (|x| is capped so that an infinite x meets its zero tail as 0 * finite: gelu(+-inf) = +inf, 0)
__device__ __forceinline__ float gelu_epi_f(float x) { return fmaf(-fminf(fabsf(x), 3.0e38f), phi_parts(x).tail, fmaxf(x, 0.0f)); }
__device__ __forceinline__ float gelu_grad_epi_f(float x) {
  const PhiParts p = phi_parts(x);
  return fmaf(x * 0.39894228040143267794f, p.e, x < 0.0f ? p.tail : 1.0f - p.tail);
}
// The same two functions for results that are stored as bfloat16, without any transcendental: odd polynomials
// in the clamped argument (least-squares fits on Chebyshev nodes, reweighted towards the minimax solution).
//   erf(x / sqrt 2)              ~ xc * P7(xc^2),  xc = clamp(x, +-3.9): absolute error below 1.3e-4 (1e-4 of it
//                                  is the tail the clamp cuts off), i.e. below 7e-5 in Phi;
//   gelu'(x) - 1/2 = Phi(x) - 1/2 + x phi(x) ~ xc * Q9(xc^2), xc = clamp(x, +-4.5): absolute error below 1.6e-4.
// A bfloat16 result carries a relative rounding error of 2e-3; the polynomial's error is below that wherever
// |gelu(x)| > 0.05 |x| (x > -1.6) and is an absolute 2e-4 |x| in the negative tail, where |gelu(x)| < 0.1.
// Twelve and fourteen full-rate instructions instead of about fourteen plus two quarter-rate ones: the
// epilogue of a 256 x 256 tile applies this 65536 times, on compute units that otherwise wait for it.
__device__ __forceinline__ float gelu_epi_bf16_f(float x) {
  const float xc = fminf(fmaxf(x, -3.9f), 3.9f), t = xc * xc;
  float p = fmaf(t, -3.635162633e-09f, 2.689292460e-07f);
  p = fmaf(t, p, -8.747332019e-06f);
  p = fmaf(t, p, 1.672272863e-04f);
  p = fmaf(t, p, -2.130134647e-03f);
  p = fmaf(t, p, 1.942755168e-02f);
  p = fmaf(t, p, -1.324737437e-01f);
  p = fmaf(t, p, 7.977387843e-01f);
  const float hx = 0.5f * x;
  return fmaf(hx, xc * p, hx);                 // x / 2 * (1 + erf(x / sqrt 2))
}
__device__ __forceinline__ float gelu_grad_epi_bf16_f(float x) {
  const float xc = fminf(fmaxf(x, -4.5f), 4.5f), t = xc * xc;
  float q = fmaf(t, -2.210824550e-11f, 2.521338996e-09f);
  q = fmaf(t, q, -1.268061318e-07f);
  q = fmaf(t, q, 3.721950556e-06f);
  q = fmaf(t, q, -7.122213527e-05f);
  q = fmaf(t, q, 9.405429872e-04f);
  q = fmaf(t, q, -8.815861893e-03f);
  q = fmaf(t, q, 5.860930499e-02f);
  q = fmaf(t, q, -2.649256748e-01f);
  q = fmaf(t, q, 7.976261395e-01f);
  return fmaf(xc, q, 0.5f);
}
__device__ __forceinline__ float sigmoid_f(float x) { return 1.0f / (1.0f + expf(-x)); }

// Wave-wide (64 lanes) sum / max by butterfly exchange.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
#endif  // __HIPCC__

}  // namespace chn
