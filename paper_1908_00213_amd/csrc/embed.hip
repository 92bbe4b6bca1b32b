// chn_embed_fwd / chn_embed_bwd: row gather by integer index (the ndarray layer's array indexing,
// Section "GPU Support by CuPy", as the language-model workload uses it) and its gradient.
//
// Forward: one wave copies one row (bit-exact), 16-byte chunks when the rows are aligned.
// Backward is written as a gather so that it needs no atomics and no workspace and is
// bit-reproducible: one block owns eight neighbouring table rows, scans the id list 256 ids at a time
// (wave ballots give each wave's matches as a bit mask), and adds the matching rows of dout to the
// table row they belong to in increasing token order.  Rows nobody referenced are written as zeros (or left alone when accumulating).
#include "common.h"

namespace chn {
namespace {

template <typename T, typename L, bool VEC>
__global__ __launch_bounds__(256) void embed_fwd_kernel(const T *table, int64_t tpitch, int64_t V, const L *ids, int64_t N, int64_t D,
                                                        T *out, int64_t opitch) {
  const int lane = threadIdx.x & 63;
  const int64_t n = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (n >= N) return;
  const int64_t id = (int64_t)ids[n];
  T *dst = out + n * opitch;
  if ((uint64_t)id >= (uint64_t)V) {   // an id outside the table is never used as an offset: its row reads as zeros
    for (int64_t d = lane; d < D; d += 64) dst[d] = T(0);
    return;
  }
  const T *src = table + id * tpitch;
  if constexpr (VEC) {
    constexpr int NV = 16 / sizeof(T);
    const int64_t nvec = D / NV;
    for (int64_t v = lane; v < nvec; v += 64)
      *reinterpret_cast<uint4 *>(dst + v * NV) = *reinterpret_cast<const uint4 *>(src + v * NV);
    for (int64_t d = nvec * NV + lane; d < D; d += 64) dst[d] = src[d];
  } else {
    for (int64_t d = lane; d < D; d += 64) dst[d] = src[d];
  }
}

constexpr int kColsPerThread = 4;
constexpr int kRowsPerBlock = 8;     // table rows one block owns: the id list is scanned once for all of them

template <typename L>
__global__ __launch_bounds__(256) void embed_bwd_kernel(const L *ids, int64_t N, const float *dout, int64_t dpitch, int64_t D,
                                                        float *dtable, int64_t tpitch, int64_t V, int accumulate) {
  __shared__ unsigned long long masks[4];
  __shared__ unsigned char which[256];           // for a matching token: which of the block's rows
  const int64_t v0 = (int64_t)blockIdx.x * kRowsPerBlock;
  const int64_t col0 = (int64_t)blockIdx.y * (256 * kColsPerThread) + threadIdx.x;
  float acc[kRowsPerBlock][kColsPerThread];
#pragma unroll
  for (int r = 0; r < kRowsPerBlock; ++r)
#pragma unroll
    for (int k = 0; k < kColsPerThread; ++k) acc[r][k] = 0.0f;
  for (int64_t base = 0; base < N; base += 256) {
    const int64_t n = base + threadIdx.x;
    const int64_t d = n < N ? (int64_t)ids[n] - v0 : -1;
    const bool hit = d >= 0 && d < kRowsPerBlock;
    const unsigned long long m = __ballot(hit);
    if ((threadIdx.x & 63) == 0) masks[threadIdx.x >> 6] = m;
    which[threadIdx.x] = (unsigned char)(hit ? d : 0);
    __syncthreads();
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      unsigned long long mm = masks[w];
      while (mm) {                                // matches in increasing token order
        const int b = __ffsll((long long)mm) - 1;
        mm &= mm - 1;
        const float *row = dout + (base + w * 64 + b) * dpitch;
        float x[kColsPerThread];
#pragma unroll
        for (int k = 0; k < kColsPerThread; ++k) {
          const int64_t c = col0 + (int64_t)k * 256;
          x[k] = c < D ? row[c] : 0.0f;
        }
        const int r_hit = which[w * 64 + b];      // uniform over the block
#pragma unroll
        for (int r = 0; r < kRowsPerBlock; ++r)
          if (r == r_hit) {
#pragma unroll
            for (int k = 0; k < kColsPerThread; ++k) acc[r][k] += x[k];
          }
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int r = 0; r < kRowsPerBlock; ++r) {
    if (v0 + r >= V) break;
#pragma unroll
    for (int k = 0; k < kColsPerThread; ++k) {
      const int64_t c = col0 + (int64_t)k * 256;
      if (c < D) {
        float *q = dtable + (v0 + r) * tpitch + c;
        *q = accumulate ? *q + acc[r][k] : acc[r][k];
      }
    }
  }
}

chn_status check_ids(const chn_array *ids, int64_t *N) {
  CHN_TRY(validate(ids, "ids", false));
  if (!is_index(ids->dtype)) return fail(CHN_ERR_DTYPE, "embed: ids must be I32 or I64");
  if (ids->ndim != 1 || !is_contiguous(ids)) return fail(CHN_ERR_SHAPE, "embed: ids must be a contiguous 1-d array");
  *N = ids->shape[0];
  return CHN_OK;
}

}  // namespace
}  // namespace chn

extern "C" {

chn_status chn_embed_fwd(const chn_array *table, const chn_array *ids, const chn_array *out, chn_stream stream) {
  using namespace chn;
  int64_t N, V, D, tp, on, od, op;
  CHN_TRY(check_ids(ids, &N));
  CHN_TRY(validate(table, "table", false));
  CHN_TRY(validate(out, "out", true));
  if (!is_float(table->dtype) || out->dtype != table->dtype) return fail(CHN_ERR_DTYPE, "embed: table and out must share F32 or BF16");
  CHN_TRY(row_major_2d(table, "table", &V, &D, &tp));
  CHN_TRY(row_major_2d(out, "out", &on, &od, &op));
  if (on != N || od != D) return fail(CHN_ERR_SHAPE, "embed: out must have shape (%lld,%lld)", (long long)N, (long long)D);
  if (N == 0 || D == 0) return CHN_OK;
  if (V == 0) return fail(CHN_ERR_SHAPE, "embed: empty table");
  const int isz = dtype_size(table->dtype);
  const bool vec = reinterpret_cast<uintptr_t>(table->data) % 16 == 0 && reinterpret_cast<uintptr_t>(out->data) % 16 == 0 &&
                   (tp * isz) % 16 == 0 && (op * isz) % 16 == 0;
  const unsigned blocks = (unsigned)((N + 3) / 4);
  hipStream_t st = as_stream(stream);
  const bool i32 = ids->dtype == CHN_I32;
#define CHN_GO(T, L, V_)                                                                                     \
  hipLaunchKernelGGL((embed_fwd_kernel<T, L, V_>), dim3(blocks), dim3(256), 0, st, static_cast<const T *>(table->data), tp, V, \
                     static_cast<const L *>(ids->data), N, D, static_cast<T *>(out->data), op)
  if (isz == 4) {
    if (i32) { if (vec) CHN_GO(float, int32_t, true); else CHN_GO(float, int32_t, false); }
    else { if (vec) CHN_GO(float, int64_t, true); else CHN_GO(float, int64_t, false); }
  } else {
    if (i32) { if (vec) CHN_GO(bf16_raw, int32_t, true); else CHN_GO(bf16_raw, int32_t, false); }
    else { if (vec) CHN_GO(bf16_raw, int64_t, true); else CHN_GO(bf16_raw, int64_t, false); }
  }
#undef CHN_GO
  return check_launch("embed_fwd");
}

chn_status chn_embed_bwd(const chn_array *ids, const chn_array *dout, const chn_array *dtable,
                         int accumulate, chn_stream stream) {
  using namespace chn;
  int64_t N, V, D, tp, dn, dd, dp;
  CHN_TRY(check_ids(ids, &N));
  CHN_TRY(validate(dout, "dout", false));
  CHN_TRY(validate(dtable, "dtable", true));
  if (dout->dtype != CHN_F32 || dtable->dtype != CHN_F32) return fail(CHN_ERR_DTYPE, "embed: dout and dtable must be F32");
  CHN_TRY(row_major_2d(dtable, "dtable", &V, &D, &tp));
  CHN_TRY(row_major_2d(dout, "dout", &dn, &dd, &dp));
  if (dn != N || dd != D) return fail(CHN_ERR_SHAPE, "embed: dout must have shape (%lld,%lld)", (long long)N, (long long)D);
  if (V == 0 || D == 0) return CHN_OK;
  if (V > 0x7fffffff) return fail(CHN_ERR_SHAPE, "embed: table too large");
  dim3 grid((unsigned)((V + kRowsPerBlock - 1) / kRowsPerBlock), (unsigned)((D + 256 * kColsPerThread - 1) / (256 * kColsPerThread)));
  if (grid.y > 65535) return fail(CHN_ERR_SHAPE, "embed: rows too wide");
  hipStream_t st = as_stream(stream);
  if (ids->dtype == CHN_I32)
    hipLaunchKernelGGL((embed_bwd_kernel<int32_t>), grid, dim3(256), 0, st, static_cast<const int32_t *>(ids->data), N,
                       static_cast<const float *>(dout->data), dp, D, static_cast<float *>(dtable->data), tp, V, accumulate);
  else
    hipLaunchKernelGGL((embed_bwd_kernel<int64_t>), grid, dim3(256), 0, st, static_cast<const int64_t *>(ids->data), N,
                       static_cast<const float *>(dout->data), dp, D, static_cast<float *>(dtable->data), tp, V, accumulate);
  return check_launch("embed_bwd");
}

}  // extern "C"
