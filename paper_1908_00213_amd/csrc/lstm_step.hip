// chn_lstm_step_fwd / chn_lstm_step_bwd: one time step of the recurrent layer in one launch.
//
// Unfused, a step is a small product (batch x 4H x H forward, batch x H x 4H backward), the kernel
// that adds its partial sums, and the point-wise cell kernel: three dependent launches of a few
// microseconds each, 35 times per direction.  The product is far too small to fill the chip, so the
// step is bound by launch latency, not by arithmetic.  Here a workgroup owns a 32 x 32 tile of the
// product -- 32 batch rows by 8 hidden units x 4 gates forward, 32 batch rows by 32 hidden units
// backward -- the operand rows stream through LDS (they are L2-resident: h and the recurrent matrix
// are re-read by every tile), its four waves take a quarter of every chunk each on the matrix cores,
// the partial tiles meet in LDS, and the same threads apply the cell.
//
// Operand layout: lane (r = lane & 31, q = lane >> 5) of a 32x32 MFMA holds row r of the tile and a
// 16-byte piece of the contraction (8 bf16 values for one 32x32x16 instruction; 4 fp32 values for four
// 32x32x2 instructions, which permutes the order of the sum but visits every term once).  Both
// operands must therefore be unit-stride along the contraction: h and dz are, and so is the recurrent
// matrix U (H, 4H) for the backward; the forward reads its transpose Ut (4H, H), which the caller
// refreshes once per optimiser step.
#include "common.h"

namespace chn {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;

template <typename T>
__device__ __forceinline__ void mma_piece(floatx16 &acc, const uint4 &a, const uint4 &b) {
  if constexpr (sizeof(T) == 2) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
  } else {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float((&a.x)[kk]), __uint_as_float((&b.x)[kk]), acc, 0, 0, 0);
  }
}

// ---- the contraction: 32 rows of A and 32 rows of B, both unit-stride along k ------------------------
// Loading the MFMA pieces straight from global memory makes every wave instruction touch 32 cache
// lines for 1 KB of data.  So the rows travel through LDS: a chunk is 512 bytes of each of the 64
// rows, copied by direct global-to-LDS loads -- two rows per wave instruction, eight whole cache lines
// -- into one of two stages while the matrix cores work on the other.  A row lies in LDS as it lies in
// memory except that its 32 16-byte pieces are permuted: piece c of row r sits at position
// c ^ (r & 15), so that the 16 lanes that read the same piece of 16 neighbouring rows together hit 16
// different bank groups.  The permutation is applied by the copying lane (position p fetches piece
// p ^ (r & 15): the same cache lines, in another lane order).
// LDS per workgroup: stages of 32 KB; the partial tiles of the four waves reuse the first stage.
// Forward: two stages, 64 KB, so two workgroups share a compute unit and a grid of 336 tiles runs in
// one round.  Backward (a four times longer contraction on a quarter of the tiles, one workgroup per
// compute unit): four stages.
constexpr int kRowBytes = 512, kStageBytes = 64 * kRowBytes;     // 8 copies per wave and stage

template <typename T, class RowA, class RowB>
__device__ __forceinline__ void copy_chunk(char *stage, RowA row_a, RowB row_b, int64_t k_len, int chunk, int wave, int lane) {
  const int64_t k0_bytes = (int64_t)chunk * kRowBytes;
  const int64_t remain = k_len * (int64_t)sizeof(T) - k0_bytes;         // bytes of the row left from this chunk on
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int pair = wave + 4 * (i & 3);                                // rows 2 * pair and 2 * pair + 1; A for i < 4, then B
    const int row = 2 * pair + (lane >> 5);
    const char *g = (i < 4 ? row_a(row) : row_b(row)) + k0_bytes;
    int64_t off = (int64_t)(((lane & 31) ^ (row & 15)) << 4);
    if (off >= remain) off = 0;                                         // past the end of the row: any valid piece, never read
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(g + off),
                                     (__attribute__((address_space(3))) void *)(stage + ((i < 4 ? 0 : 32) + 2 * pair) * kRowBytes),
                                     16, 0, 0);
  }
}

// This wave's quarter of the 32-byte slices of one staged chunk.
template <typename T>
__device__ __forceinline__ void mma_chunk(floatx16 &acc, const char *stage, int n_slices, int wave, int lane) {
  const int r = lane & 31, q = lane >> 5;
  const char *pa = stage + r * kRowBytes, *pb = stage + (32 + r) * kRowBytes;
  uint4 a[4], b[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int s = wave * 4 + u;
    if (s < n_slices) {                       // uniform over the wave
      const int pos = ((2 * s + q) ^ (r & 15)) << 4;
      a[u] = *reinterpret_cast<const uint4 *>(pa + pos);
      b[u] = *reinterpret_cast<const uint4 *>(pb + pos);
    }
  }
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (wave * 4 + u < n_slices) mma_piece<T>(acc, a[u], b[u]);
}

// acc (this wave's partial tile) = sum over k of A[row r of the tile][k] * B[row r][k] for this
// wave's share of k.  row_a(i) / row_b(i) give the global address of row i (0..31) of each operand.
// NS stages, NS separate LDS arrays, the loop written out for every role of each: only then can the
// compiler tell that a copy in flight into one does not concern the reads of another.  A chunk is
// consumed in far less time than it takes to arrive, so the rate is set by the bytes in flight:
// NS chunks per workgroup.  On return every wave has passed a barrier after its last read.
template <typename T, int NS, class RowA, class RowB>
__device__ __forceinline__ void contract(floatx16 &acc, char *const (&stages)[NS], RowA row_a, RowB row_b, int64_t k_len, int wave, int lane) {
  static_assert(NS >= 2 && NS <= 4, "the wait immediates below cover up to three chunks in flight behind the current one");
  constexpr int kSliceElems = 32 / (int)sizeof(T), kChunkElems = kRowBytes / (int)sizeof(T);
  const int n_chunks = (int)((k_len + kChunkElems - 1) / kChunkElems);
#pragma unroll
  for (int k = 0; k < NS; ++k)
    if (k < n_chunks) copy_chunk<T>(stages[k], row_a, row_b, k_len, k, wave, lane);
  auto step = [&](char *cur, int ch) {
    // the copies of chunk ch are older than those of the chunks behind it, which may stay in flight
    // (8 copies per wave and chunk; s_waitcnt immediates that name vmcnt only)
    const int behind = n_chunks - 1 - ch < NS - 1 ? n_chunks - 1 - ch : NS - 1;
    if (behind == 0) __builtin_amdgcn_s_waitcnt(0x0F70);
    else if (behind == 1) __builtin_amdgcn_s_waitcnt(0x0F78);
    else if (behind == 2) __builtin_amdgcn_s_waitcnt(0x4F70);
    else __builtin_amdgcn_s_waitcnt(0x4F78);
    // Plain barriers with explicit waits instead of __syncthreads(): its fence would wait for every
    // copy in flight, also those of the chunks behind, and the pipeline would be one chunk deep.
    // What the first barrier publishes is this wave's copies of chunk ch (waited for above); what the
    // second one protects is `cur`, which may be overwritten once every wave's LDS reads have
    // returned (waited for below).
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    const int64_t left = k_len - (int64_t)ch * kChunkElems;
    mma_chunk<T>(acc, cur, (int)((left < kChunkElems ? left : kChunkElems) / kSliceElems), wave, lane);
    __builtin_amdgcn_s_waitcnt(0xC07F);       // lgkmcnt(0): the fragment reads have returned
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (ch + NS < n_chunks) copy_chunk<T>(cur, row_a, row_b, k_len, ch + NS, wave, lane);
  };
  for (int ch = 0; ch < n_chunks; ch += NS) {
#pragma unroll
    for (int k = 0; k < NS; ++k)
      if (ch + k < n_chunks) step(stages[k], ch + k);
  }
}

// The same contraction with ONE barrier per chunk, for long contractions on few tiles (the backward
// step).  A wave that has passed the barrier of chunk ch has finished reading chunk ch - 1, so the
// stage of chunk ch - 1 can be refilled right behind that barrier and no second barrier is needed;
// the price is one stage that is neither being read nor in flight, i.e. NS - 1 chunks of look-ahead.
template <typename T, int NS, class RowA, class RowB>
__device__ __forceinline__ void contract_long(floatx16 &acc, char *const (&stages)[NS], RowA row_a, RowB row_b, int64_t k_len, int wave, int lane) {
  static_assert(NS == 4, "the wait immediates below are written for four stages");
  constexpr int kSliceElems = 32 / (int)sizeof(T), kChunkElems = kRowBytes / (int)sizeof(T);
  const int n_chunks = (int)((k_len + kChunkElems - 1) / kChunkElems);
#pragma unroll
  for (int k = 0; k < NS - 1; ++k)
    if (k < n_chunks) copy_chunk<T>(stages[k], row_a, row_b, k_len, k, wave, lane);
  auto step = [&](char *cur, char *refill, int ch) {
    // issued so far: chunks 0 .. ch + NS - 2; those behind chunk ch may stay in flight
    const int behind = n_chunks - 1 - ch < NS - 2 ? n_chunks - 1 - ch : NS - 2;
    if (behind == 0) __builtin_amdgcn_s_waitcnt(0x0070);        // vmcnt(0) lgkmcnt(0)
    else if (behind == 1) __builtin_amdgcn_s_waitcnt(0x0078);   // vmcnt(8) lgkmcnt(0)
    else __builtin_amdgcn_s_waitcnt(0x4070);                    // vmcnt(16) lgkmcnt(0)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (ch + NS - 1 < n_chunks) copy_chunk<T>(refill, row_a, row_b, k_len, ch + NS - 1, wave, lane);
    const int64_t left = k_len - (int64_t)ch * kChunkElems;
    mma_chunk<T>(acc, cur, (int)((left < kChunkElems ? left : kChunkElems) / kSliceElems), wave, lane);
  };
  for (int ch = 0; ch < n_chunks; ch += NS) {
#pragma unroll
    for (int k = 0; k < NS; ++k)
      if (ch + k < n_chunks) step(stages[k], stages[(k + NS - 1) % NS], ch + k);
  }
  __builtin_amdgcn_s_waitcnt(0xC07F);         // lgkmcnt(0): the last fragment reads have returned
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Park this wave's partial tile in LDS as tile[wave][row][col]: lane (r, q) holds column r and the
// rows 8 * (v / 4) + 4 * q + v % 4 of its 16 accumulators.
__device__ __forceinline__ void park(float (*tile)[32][33], const floatx16 &acc, int wave, int lane) {
  const int r = lane & 31, q = lane >> 5;
#pragma unroll
  for (int v = 0; v < 16; ++v) tile[wave][8 * (v / 4) + 4 * q + v % 4][r] = acc[v];
}

__device__ __forceinline__ float total(float (*tile)[32][33], int row, int col) {
  return (tile[0][row][col] + tile[1][row][col]) + (tile[2][row][col] + tile[3][row][col]);
}

static_assert(sizeof(float) * kWaves * 32 * 33 <= kStageBytes, "the partial tiles must fit into one stage");

struct FwdArgs {
  int64_t B, H;
  const float *zx; int64_t zx_pitch;
  const void *h_prev; int64_t hp_pitch;
  const void *Ut; int64_t ut_pitch;
  const float *bias;
  const float *c_prev; int64_t cp_pitch;
  float *c; int64_t c_pitch;
  void *h; int64_t h_pitch;
  float *gates; int64_t g_pitch;
};

// grid: (H / 8, ceil(B / 32)).  Tile column 8 * g + jj is gate g of hidden unit j0 + jj.
template <typename T>
__global__ __launch_bounds__(kThreads) void lstm_step_fwd_kernel(FwdArgs a) {
  __shared__ __attribute__((aligned(1024))) char stage0[kStageBytes];
  __shared__ __attribute__((aligned(1024))) char stage1[kStageBytes];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t j0 = (int64_t)blockIdx.x * 8, b0 = (int64_t)blockIdx.y * 32;
  // this thread's (batch row, hidden unit) pair of the cell; its inputs are fetched now, so that
  // their latency passes under the contraction
  const int row = threadIdx.x >> 3, jj = threadIdx.x & 7;
  const int64_t b = b0 + row, j = j0 + jj;
  const bool live = b < a.B;
  float z[4] = {0.0f, 0.0f, 0.0f, 0.0f}, cp = 0.0f;
  if (live) {
    const float *zr = a.zx + b * a.zx_pitch;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      z[g] = zr[g * a.H + j];
      if (a.bias) z[g] += a.bias[g * a.H + j];
    }
    cp = a.c_prev[b * a.cp_pitch + j];
  }
  auto row_a = [&](int i) {                                        // rows past the batch repeat the last one
    const int64_t bb = b0 + i < a.B ? b0 + i : a.B - 1;
    return reinterpret_cast<const char *>(static_cast<const T *>(a.h_prev) + bb * a.hp_pitch);
  };
  auto row_b = [&](int i) {                                        // tile column i = gate i / 8 of unit j0 + i % 8
    return reinterpret_cast<const char *>(static_cast<const T *>(a.Ut) + ((int64_t)(i >> 3) * a.H + j0 + (i & 7)) * a.ut_pitch);
  };
  floatx16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
  char *const stages[2] = {stage0, stage1};
  contract<T, 2>(acc, stages, row_a, row_b, a.H, wave, lane);
  float (*tile)[32][33] = reinterpret_cast<float (*)[32][33]>(stage0);
  park(tile, acc, wave, lane);
  __syncthreads();
  if (!live) return;
#pragma unroll
  for (int g = 0; g < 4; ++g) z[g] += total(tile, row, 8 * g + jj);
  const float i = sigmoid_f(z[0]), f = sigmoid_f(z[1]), g = tanhf(z[2]), o = sigmoid_f(z[3]);
  const float cn = f * cp + i * g;
  a.c[b * a.c_pitch + j] = cn;
  Elem<T>::store(static_cast<T *>(a.h) + b * a.h_pitch + j, o * tanhf(cn));
  if (a.gates) {
    float *gr = a.gates + b * a.g_pitch;
    gr[j] = i; gr[a.H + j] = f; gr[2 * a.H + j] = g; gr[3 * a.H + j] = o;
  }
}

struct BwdArgs {
  int64_t B, H;
  const void *dz_next; int64_t dzn_pitch;      // NULL: no later step
  const void *U; int64_t u_pitch;
  void *dh; int64_t dh_pitch;                  // in: the part from the layers above; out: the total
  const float *gates; int64_t g_pitch;
  const float *c_prev; int64_t cp_pitch;
  const float *c; int64_t c_pitch;
  const float *dc_next; int64_t dcn_pitch;
  void *dz; int64_t dz_pitch;
  float *dc_prev; int64_t dcp_pitch;
};

// grid: (H / 32, ceil(B / 32)).  dh[b, j] += sum_k dz_next[b, k] U[j, k], then the cell's backward.
template <typename T>
__global__ __launch_bounds__(kThreads) void lstm_step_bwd_kernel(BwdArgs a) {
  __shared__ __attribute__((aligned(1024))) char stage0[kStageBytes];
  __shared__ __attribute__((aligned(1024))) char stage1[kStageBytes];
  __shared__ __attribute__((aligned(1024))) char stage2[kStageBytes];
  __shared__ __attribute__((aligned(1024))) char stage3[kStageBytes];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t j0 = (int64_t)blockIdx.x * 32, b0 = (int64_t)blockIdx.y * 32;
  // four (batch row, hidden unit) pairs per thread, neighbouring threads on neighbouring units; what
  // the cell's backward reads is fetched now, so that its latency passes under the contraction
  const int col = threadIdx.x & 31;
  const int64_t j = j0 + col;
  float dh[4], gi[4], gf[4], gg[4], go[4], cc[4], cp[4], dcn[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int64_t b = b0 + (threadIdx.x >> 5) + 8 * p;
    dh[p] = gi[p] = gf[p] = gg[p] = go[p] = cc[p] = cp[p] = dcn[p] = 0.0f;
    if (b < a.B) {
      dh[p] = Elem<T>::load(static_cast<const T *>(a.dh) + b * a.dh_pitch + j);
      const float *gr = a.gates + b * a.g_pitch;
      gi[p] = gr[j]; gf[p] = gr[a.H + j]; gg[p] = gr[2 * a.H + j]; go[p] = gr[3 * a.H + j];
      cc[p] = a.c[b * a.c_pitch + j];
      cp[p] = a.c_prev[b * a.cp_pitch + j];
      if (a.dc_next) dcn[p] = a.dc_next[b * a.dcn_pitch + j];
    }
  }
  float (*tile)[32][33] = reinterpret_cast<float (*)[32][33]>(stage0);
  if (a.dz_next) {
    auto row_a = [&](int i) {
      const int64_t bb = b0 + i < a.B ? b0 + i : a.B - 1;
      return reinterpret_cast<const char *>(static_cast<const T *>(a.dz_next) + bb * a.dzn_pitch);
    };
    auto row_b = [&](int i) { return reinterpret_cast<const char *>(static_cast<const T *>(a.U) + (j0 + i) * a.u_pitch); };
    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
    char *const stages[4] = {stage0, stage1, stage2, stage3};
    contract_long<T, 4>(acc, stages, row_a, row_b, 4 * a.H, wave, lane);
    park(tile, acc, wave, lane);
    __syncthreads();
  }
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int row = (threadIdx.x >> 5) + 8 * p;
    const int64_t b = b0 + row;
    if (b >= a.B) continue;
    float d = dh[p];
    if (a.dz_next) {
      // the total is what the cell sees and what is stored: in mixed precision that is the bf16 value
      d += total(tile, row, col);
      Elem<T>::store(static_cast<T *>(a.dh) + b * a.dh_pitch + j, d);
      if constexpr (sizeof(T) == 2) d = bf16_to_f32(f32_to_bf16(d));
    }
    const float i = gi[p], f = gf[p], g = gg[p], o = go[p];
    const float tc = tanhf(cc[p]);
    const float d_o = d * tc;
    const float dc = dcn[p] + d * o * (1.0f - tc * tc);
    const float di = dc * g, dg = dc * i, df = dc * cp[p];
    a.dc_prev[b * a.dcp_pitch + j] = dc * f;
    T *dr = static_cast<T *>(a.dz) + b * a.dz_pitch;
    Elem<T>::store(dr + j, di * i * (1.0f - i));
    Elem<T>::store(dr + a.H + j, df * f * (1.0f - f));
    Elem<T>::store(dr + 2 * a.H + j, dg * (1.0f - g * g));
    Elem<T>::store(dr + 3 * a.H + j, d_o * o * (1.0f - o));
  }
}

// (rows, cols) view with unit inner stride; `t` (F32 or BF16) or F32 only; optionally rows that
// start on 16-byte boundaries (operands of the contraction)
chn_status view(const chn_array *x, const char *name, bool out, int64_t rows, int64_t cols, int want_dtype, bool operand,
                int64_t *pitch) {
  CHN_TRY(validate(x, name, out));
  if (x->dtype != want_dtype)
    return fail(CHN_ERR_DTYPE, "lstm_step: %s must be %s", name, want_dtype == CHN_F32 ? "F32" : "BF16");
  int64_t r, c;
  CHN_TRY(row_major_2d(x, name, &r, &c, pitch));
  if (r != rows || c != cols)
    return fail(CHN_ERR_SHAPE, "lstm_step: %s must have shape (%lld,%lld)", name, (long long)rows, (long long)cols);
  if (operand) {
    const int per16 = 16 / dtype_size(x->dtype);
    if (reinterpret_cast<uintptr_t>(x->data) % 16 || (rows > 1 && *pitch % per16))
      return fail(CHN_ERR_STRIDE, "lstm_step: rows of %s must start on 16-byte boundaries", name);
  }
  return CHN_OK;
}

}  // namespace
}  // namespace chn

extern "C" {

chn_status chn_lstm_step_fwd(const chn_array *zx, const chn_array *h_prev, const chn_array *Ut, const chn_array *bias,
                             const chn_array *c_prev, const chn_array *c, const chn_array *h, const chn_array *gates,
                             chn_stream stream) {
  using namespace chn;
  CHN_TRY(validate(c_prev, "c_prev", false));
  if (c_prev->ndim != 2) return fail(CHN_ERR_NDIM, "lstm_step: c_prev must be 2-d");
  if (!h_prev) return fail(CHN_ERR_NULL, "lstm_step: h_prev is NULL");
  FwdArgs a{};
  a.B = c_prev->shape[0]; a.H = c_prev->shape[1];
  if (a.H % 32) return fail(CHN_ERR_SHAPE, "lstm_step: the hidden width %lld is not a multiple of 32 (pad it, or use the unfused calls)", (long long)a.H);
  const int t = h_prev->dtype;
  if (t != CHN_F32 && t != CHN_BF16) return fail(CHN_ERR_DTYPE, "lstm_step: h_prev must be F32 or BF16");
  CHN_TRY(view(c_prev, "c_prev", false, a.B, a.H, CHN_F32, false, &a.cp_pitch));
  CHN_TRY(view(zx, "zx", false, a.B, 4 * a.H, CHN_F32, false, &a.zx_pitch));
  CHN_TRY(view(h_prev, "h_prev", false, a.B, a.H, t, true, &a.hp_pitch));
  CHN_TRY(view(Ut, "Ut", false, 4 * a.H, a.H, t, true, &a.ut_pitch));
  CHN_TRY(view(c, "c", true, a.B, a.H, CHN_F32, false, &a.c_pitch));
  CHN_TRY(view(h, "h", true, a.B, a.H, t, false, &a.h_pitch));
  if (gates) CHN_TRY(view(gates, "gates", true, a.B, 4 * a.H, CHN_F32, false, &a.g_pitch));
  if (bias) {
    CHN_TRY(validate(bias, "bias", false));
    if (bias->dtype != CHN_F32 || bias->ndim != 1 || bias->shape[0] != 4 * a.H || !is_contiguous(bias))
      return fail(CHN_ERR_SHAPE, "lstm_step: bias must be a contiguous F32 (%lld,) array", (long long)(4 * a.H));
  }
  if (a.B * a.H == 0) return CHN_OK;
  const int64_t by = (a.B + 31) / 32;
  if (by > 65535) return fail(CHN_ERR_SHAPE, "lstm_step: batch too large");
  a.zx = static_cast<const float *>(zx->data);
  a.h_prev = h_prev->data; a.Ut = Ut->data;
  a.bias = bias ? static_cast<const float *>(bias->data) : nullptr;
  a.c_prev = static_cast<const float *>(c_prev->data);
  a.c = static_cast<float *>(c->data);
  a.h = h->data;
  a.gates = gates ? static_cast<float *>(gates->data) : nullptr;
  const dim3 grid((unsigned)(a.H / 8), (unsigned)by);
  if (t == CHN_BF16) hipLaunchKernelGGL(lstm_step_fwd_kernel<bf16_raw>, grid, dim3(kThreads), 0, as_stream(stream), a);
  else hipLaunchKernelGGL(lstm_step_fwd_kernel<float>, grid, dim3(kThreads), 0, as_stream(stream), a);
  return check_launch("lstm_step_fwd");
}

chn_status chn_lstm_step_bwd(const chn_array *dz_next, const chn_array *U, const chn_array *dh, const chn_array *gates,
                             const chn_array *c_prev, const chn_array *c, const chn_array *dc_next, const chn_array *dz,
                             const chn_array *dc_prev, chn_stream stream) {
  using namespace chn;
  CHN_TRY(validate(c, "c", false));
  if (c->ndim != 2) return fail(CHN_ERR_NDIM, "lstm_step: c must be 2-d");
  if (!dh) return fail(CHN_ERR_NULL, "lstm_step: dh is NULL");
  BwdArgs a{};
  a.B = c->shape[0]; a.H = c->shape[1];
  if (a.H % 32) return fail(CHN_ERR_SHAPE, "lstm_step: the hidden width %lld is not a multiple of 32 (pad it, or use the unfused calls)", (long long)a.H);
  const int t = dh->dtype;
  if (t != CHN_F32 && t != CHN_BF16) return fail(CHN_ERR_DTYPE, "lstm_step: dh must be F32 or BF16");
  CHN_TRY(view(c, "c", false, a.B, a.H, CHN_F32, false, &a.c_pitch));
  CHN_TRY(view(c_prev, "c_prev", false, a.B, a.H, CHN_F32, false, &a.cp_pitch));
  CHN_TRY(view(gates, "gates", false, a.B, 4 * a.H, CHN_F32, false, &a.g_pitch));
  CHN_TRY(view(dh, "dh", true, a.B, a.H, t, false, &a.dh_pitch));
  if (dz_next) {
    CHN_TRY(view(dz_next, "dz_next", false, a.B, 4 * a.H, t, true, &a.dzn_pitch));
    CHN_TRY(view(U, "U", false, a.H, 4 * a.H, t, true, &a.u_pitch));
  }
  if (dc_next) CHN_TRY(view(dc_next, "dc_next", false, a.B, a.H, CHN_F32, false, &a.dcn_pitch));
  CHN_TRY(view(dz, "dz", true, a.B, 4 * a.H, t, false, &a.dz_pitch));
  CHN_TRY(view(dc_prev, "dc_prev", true, a.B, a.H, CHN_F32, false, &a.dcp_pitch));
  if (a.B * a.H == 0) return CHN_OK;
  const int64_t by = (a.B + 31) / 32;
  if (by > 65535) return fail(CHN_ERR_SHAPE, "lstm_step: batch too large");
  a.dz_next = dz_next ? dz_next->data : nullptr;
  a.U = dz_next ? U->data : nullptr;
  a.dh = dh->data;
  a.gates = static_cast<const float *>(gates->data);
  a.c_prev = static_cast<const float *>(c_prev->data);
  a.c = static_cast<const float *>(c->data);
  a.dc_next = dc_next ? static_cast<const float *>(dc_next->data) : nullptr;
  a.dz = dz->data;
  a.dc_prev = static_cast<float *>(dc_prev->data);
  const dim3 grid((unsigned)(a.H / 32), (unsigned)by);
  if (t == CHN_BF16) hipLaunchKernelGGL(lstm_step_bwd_kernel<bf16_raw>, grid, dim3(kThreads), 0, as_stream(stream), a);
  else hipLaunchKernelGGL(lstm_step_bwd_kernel<float>, grid, dim3(kThreads), 0, as_stream(stream), a);
  return check_launch("lstm_step_bwd");
}

}  // extern "C"
