// chn_argmax_axis: index of the largest element along one axis (the classification example of Section
// "API Design" reports accuracy, i.e. the arg-max of the logits against the labels).  Among equal
// maxima the smallest index wins (NumPy's rule); a NaN is never selected, and a slice that holds
// nothing but NaN yields index 0.
// Two shapes of work: the reduced axis has unit stride -> one wave per result, lanes stride the row
// and a butterfly picks the winner; anything else -> one thread per result (neighbouring threads on
// neighbouring results, so reads along a unit-stride kept dimension coalesce).
#include "common.h"

namespace chn {
namespace {

struct AArgs {
  const void *in; void *out;
  int nk;
  int64_t kshape[CHN_MAX_NDIM], kstr[CHN_MAX_NDIM];
  int64_t len, sR, total_out;
};

__device__ __forceinline__ bool better(float v, int64_t i, float bv, int64_t bi) {
  return v > bv || (v == bv && i < bi);
}

template <typename Tin, typename Tout, bool ROWS>
__global__ __launch_bounds__(256) void argmax_kernel(AArgs a) {
  const int lane = threadIdx.x & 63;
  int64_t e = ROWS ? (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6) : (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= a.total_out) return;
  int64_t off = 0, rem = e;
  for (int d = a.nk - 1; d >= 0; --d) { off += (rem % a.kshape[d]) * a.kstr[d]; rem /= a.kshape[d]; }
  const Tin *p = static_cast<const Tin *>(a.in) + off;
  float bv = -INFINITY;
  int64_t bi = 0x7fffffffffffffffll;
  if constexpr (ROWS) {
    for (int64_t r = lane; r < a.len; r += 64) {
      const float v = Elem<Tin>::load(p + r * a.sR);
      if (better(v, r, bv, bi)) { bv = v; bi = r; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float ov = __shfl_xor(bv, o, 64);
      const int64_t oi = __shfl_xor(bi, o, 64);
      if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    if (lane != 0) return;
  } else {
    for (int64_t r = 0; r < a.len; ++r) {
      const float v = Elem<Tin>::load(p + r * a.sR);
      if (better(v, r, bv, bi)) { bv = v; bi = r; }
    }
  }
  if (bi == 0x7fffffffffffffffll) bi = 0;       // nothing compared greater than -inf
  static_cast<Tout *>(a.out)[e] = (Tout)bi;
}

}  // namespace
}  // namespace chn

extern "C" chn_status chn_argmax_axis(const chn_array *in, int axis, int keepdims, const chn_array *out, chn_stream stream) {
  using namespace chn;
  CHN_TRY(validate(in, "in", false));
  if (!is_float(in->dtype)) return fail(CHN_ERR_DTYPE, "argmax: input must be F32 or BF16");
  if (in->ndim < 1) return fail(CHN_ERR_NDIM, "argmax: input needs at least one dimension");
  const int ax = axis < 0 ? axis + in->ndim : axis;
  if (ax < 0 || ax >= in->ndim) return fail(CHN_ERR_AXIS, "argmax: axis %d out of range for ndim %d", axis, in->ndim);
  CHN_TRY(validate(out, "out", true));
  if (!is_index(out->dtype)) return fail(CHN_ERR_DTYPE, "argmax: out must be I32 or I64");
  const int ond = keepdims ? in->ndim : in->ndim - 1;
  if (out->ndim != ond) return fail(CHN_ERR_SHAPE, "argmax: out has ndim %d, expected %d", out->ndim, ond);
  for (int d = 0, od = 0; d < in->ndim; ++d) {
    if (d == ax) {
      if (keepdims) { if (out->shape[od] != 1) return fail(CHN_ERR_SHAPE, "argmax: kept axis must have length 1"); ++od; }
      continue;
    }
    if (out->shape[od] != in->shape[d]) return fail(CHN_ERR_SHAPE, "argmax: out dimension %d has length %lld, expected %lld", od, (long long)out->shape[od], (long long)in->shape[d]);
    ++od;
  }
  if (!is_contiguous(out)) return fail(CHN_ERR_STRIDE, "argmax: out must be contiguous");
  if (in->shape[ax] == 0) return fail(CHN_ERR_SHAPE, "argmax: the reduced axis is empty");
  const int isz = dtype_size(in->dtype);
  AArgs a{};
  a.in = in->data; a.out = out->data;
  a.len = in->shape[ax];
  a.sR = a.len > 1 ? in->strides[ax] / isz : 1;
  a.total_out = 1;
  for (int d = 0; d < in->ndim; ++d) {
    if (d == ax) continue;
    a.total_out *= in->shape[d];
    if (in->shape[d] == 1) continue;
    a.kshape[a.nk] = in->shape[d];
    a.kstr[a.nk] = in->strides[d] / isz;
    ++a.nk;
  }
  if (a.total_out == 0) return CHN_OK;
  const bool rows = a.sR == 1 && a.len >= 64;
  const int64_t blocks = rows ? (a.total_out + 3) / 4 : (a.total_out + 255) / 256;
  if (blocks > 0x7fffffff) return fail(CHN_ERR_SHAPE, "argmax: too many results");
  const dim3 grid((unsigned)blocks), block(256);
  hipStream_t st = as_stream(stream);
#define CHN_ARGMAX(TI, TO)                                                                        \
  do {                                                                                            \
    if (rows) hipLaunchKernelGGL((argmax_kernel<TI, TO, true>), grid, block, 0, st, a);           \
    else hipLaunchKernelGGL((argmax_kernel<TI, TO, false>), grid, block, 0, st, a);               \
  } while (0)
  if (in->dtype == CHN_F32 && out->dtype == CHN_I64) CHN_ARGMAX(float, int64_t);
  else if (in->dtype == CHN_F32) CHN_ARGMAX(float, int32_t);
  else if (out->dtype == CHN_I64) CHN_ARGMAX(bf16_raw, int64_t);
  else CHN_ARGMAX(bf16_raw, int32_t);
#undef CHN_ARGMAX
  return check_launch("argmax");
}
