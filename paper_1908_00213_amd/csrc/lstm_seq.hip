// chn_lstm_seq_fwd: all time steps of the recurrent layer's forward pass in ONE launch.
//
// Step by step (chn_lstm_step_fwd) every launch fetches its slice of the recurrent matrix again and pays a
// launch, a pipeline ramp and a drain for 0.46 GFLOP of work.  Here the grid stays resident for the whole
// sequence: a workgroup owns 8 hidden units (the 32 gate columns i, f, g, o of those units) for 64 batch
// rows, keeps its 32 rows of Ut in LDS from the first step to the last and its cell state in registers, and
// per step streams the 64 rows of h_{t-1} through two LDS stages, multiplies on the matrix cores (each of
// the four waves a quarter of the contraction), applies the cell and publishes its 64 x 8 piece of h_t.
//
// What the workgroups exchange is h: all-to-all among the H / 8 workgroups of one batch block, every step.
// The compute units of the chip sit behind eight separate L2 caches that are coherent with each other only
// at kernel boundaries, so the exchange goes past them: h_t is written with agent-scope stores (written
// through), the arrival of a workgroup's piece is counted in one agent-scope counter per batch block, and
// h_{t-1} is read with agent-scope (sc1) direct-to-LDS loads after the counter has reached (steps so far) x
// (workgroups of the block).  Measured between 84 workgroups: 1.6-1.9 us per exchange.
//
// Every wait is bounded: a workgroup that does not see its counter arrive within `spin_limit` polls (the grid
// does not fit the device next to other work, say) raises the status word and leaves; every other workgroup
// sees the status word in its next poll and leaves too.  The kernel always ends; the caller checks the status
// word after synchronising (chn_lstm_seq_status) and falls back to the per-step calls if it is set.
#include <atomic>

#include "common.h"

namespace chn {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kThreads = 256;
constexpr int kRowBytes = 512;                         // bytes of one operand row per chunk
constexpr int kUChunkBytes = 32 * kRowBytes;           // 32 rows of Ut
constexpr int kHStageBytes = 64 * kRowBytes;           // 64 rows of h
constexpr int kMaxChunks = 6;                          // rows of up to 3072 bytes: H <= 768 (F32), 1536 (BF16)
constexpr int kCpolAgent = 17;                         // sc0 | sc1 on a direct-to-LDS load

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

struct SeqArgs {
  int64_t B, H;
  int n_steps, nub, spin_limit;
  const float *zx; int64_t zx_pitch;
  const void *Ut; int64_t ut_pitch;
  const float *bias;
  void *Hs; int64_t h_pitch;
  float *Cs; int64_t c_pitch;
  float *gates; int64_t g_pitch;
  unsigned *counters;        // one per batch block, zero at launch
  unsigned *status;          // zero at launch; 1 = a bounded wait ran out
};

__global__ __launch_bounds__(64) void seq_clear_kernel(unsigned *p, int n) {
  for (int i = threadIdx.x; i < n; i += 64) p[i] = 0u;
}

// Agent-scope store of two neighbouring values of a row of h (one 8-byte or 4-byte access).
__device__ __forceinline__ void store_h2(float *p, float v0, float v1) {
  unsigned long long bits = (unsigned long long)__float_as_uint(v0) | ((unsigned long long)__float_as_uint(v1) << 32);
  __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_h2(bf16_raw *p, float v0, float v1) {
  unsigned bits = (unsigned)f32_to_bf16(v0) | ((unsigned)f32_to_bf16(v1) << 16);
  __hip_atomic_store(reinterpret_cast<unsigned *>(p), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// grid: (H / 8, ceil(B / 64)).  Tile column 8 * g + jj is gate g of hidden unit j0 + jj.
template <typename T>
__global__ __launch_bounds__(kThreads) void lstm_seq_fwd_kernel(SeqArgs a) {
  __shared__ __attribute__((aligned(1024))) char uslice[kMaxChunks * kUChunkBytes];
  __shared__ __attribute__((aligned(1024))) char stage0[kHStageBytes];
  __shared__ __attribute__((aligned(1024))) char stage1[kHStageBytes];
  // the word in which wave 0 tells the others that a wait ran out: the tail of a stage, free between two steps
  volatile int &give_up = *reinterpret_cast<volatile int *>(stage1 + kHStageBytes - 4);
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  const int64_t j0 = (int64_t)blockIdx.x * 8, b0 = (int64_t)blockIdx.y * 64;
  const int64_t row_bytes = a.H * (int64_t)sizeof(T);
  const int n_chunks = (int)((row_bytes + kRowBytes - 1) / kRowBytes);
  // ---- the workgroup's 32 rows of Ut, once
#pragma unroll 1
  for (int ch = 0; ch < n_chunks; ++ch) {
    const int64_t remain = row_bytes - (int64_t)ch * kRowBytes;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int pair = wave + 4 * i, row = 2 * pair + (lane >> 5);
      const char *g = reinterpret_cast<const char *>(static_cast<const T *>(a.Ut) + ((int64_t)(row >> 3) * a.H + j0 + (row & 7)) * a.ut_pitch) +
                      (int64_t)ch * kRowBytes;
      int64_t off = (int64_t)(((lane & 31) ^ (row & 15)) << 4);
      if (off >= remain) off = 0;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(g + off),
                                       (__attribute__((address_space(3))) void *)(uslice + ch * kUChunkBytes + 2 * pair * kRowBytes), 16, 0, 0);
    }
  }

  // ---- this thread's part of the cell: one batch row, two neighbouring hidden units
  const int crow = threadIdx.x >> 2, jj = (threadIdx.x & 3) * 2;
  const int64_t b = b0 + crow, j = j0 + jj;
  const bool live = b < a.B;
  float c_state[2] = {0.0f, 0.0f};
  float bias[4][2];
#pragma unroll
  for (int g = 0; g < 4; ++g) { bias[g][0] = a.bias ? a.bias[g * a.H + j] : 0.0f; bias[g][1] = a.bias ? a.bias[g * a.H + j + 1] : 0.0f; }
  if (live) { c_state[0] = a.Cs[b * a.c_pitch + j]; c_state[1] = a.Cs[b * a.c_pitch + j + 1]; }
  __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0): Ut has landed
  __syncthreads();

  // copies of chunk `ch` of the 64 rows of h (block `blk` of Hs) into a stage; rows past the batch repeat the last one
  auto copy_h = [&](char *stage, const T *hblk, int ch) {
    const int64_t remain = row_bytes - (int64_t)ch * kRowBytes;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int pair = wave + 4 * i, row = 2 * pair + (lane >> 5);
      const int64_t bb = b0 + row < a.B ? b0 + row : a.B - 1;
      const char *g = reinterpret_cast<const char *>(hblk + bb * a.h_pitch) + (int64_t)ch * kRowBytes;
      int64_t off = (int64_t)(((lane & 31) ^ (row & 15)) << 4);
      if (off >= remain) off = 0;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(g + off),
                                       (__attribute__((address_space(3))) void *)(stage + 2 * pair * kRowBytes), 16, 0, kCpolAgent);
    }
  };
  // this wave's quarter of the 32-byte slices of a staged chunk, against the resident rows of Ut
  auto mma_chunk = [&](floatx16 &acc0, floatx16 &acc1, const char *stage, int ch) {
    const int64_t left = row_bytes - (int64_t)ch * kRowBytes;
    const int n_slices = (int)((left < kRowBytes ? left : kRowBytes) / 32);
    const int r = lane & 31, q = lane >> 5;
    const char *pa = stage + r * kRowBytes, *pb = uslice + ch * kUChunkBytes + r * kRowBytes;
    uint4 x0[4], x1[4], y[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int s = wave * 4 + u;
      if (s < n_slices) {
        const int pos = ((2 * s + q) ^ (r & 15)) << 4;
        x0[u] = *reinterpret_cast<const uint4 *>(pa + pos);
        x1[u] = *reinterpret_cast<const uint4 *>(pa + 32 * kRowBytes + pos);
        y[u] = *reinterpret_cast<const uint4 *>(pb + pos);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (wave * 4 + u < n_slices) { mma_piece<T>(acc0, x0[u], y[u]); mma_piece<T>(acc1, x1[u], y[u]); }
  };
  float (*tile0)[32][33] = reinterpret_cast<float (*)[32][33]>(stage0);   // partial tiles of rows 0-31 / 32-63, per wave
  float (*tile1)[32][33] = reinterpret_cast<float (*)[32][33]>(stage1);
  static_assert(sizeof(float) * 4 * 32 * 33 <= kHStageBytes, "the partial tiles of four waves fit a stage");

#pragma unroll 1
  for (int t = 0; t < a.n_steps; ++t) {
    // what the cell needs besides the product, fetched early
    float z[4][2];
    if (live) {
      const float *zr = a.zx + ((int64_t)t * a.B + b) * a.zx_pitch;
#pragma unroll
      for (int g = 0; g < 4; ++g) { z[g][0] = zr[g * a.H + j] + bias[g][0]; z[g][1] = zr[g * a.H + j + 1] + bias[g][1]; }
    }
    // ---- h_{t-1} of every workgroup of this batch block must have arrived (step 0 reads the caller's h_0)
    if (t > 0) {
      if (wave == 0) {
        const unsigned want = (unsigned)t * (unsigned)a.nub;
        bool ok = false;
        if (lane == 0) give_up = 0;
#pragma unroll 1
        for (int spins = 0; spins < a.spin_limit; ++spins) {
          const unsigned seen = __hip_atomic_load(a.counters + blockIdx.y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          const unsigned st = __hip_atomic_load(a.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          ok = seen >= want;
          if (ok || st != 0u) break;
          __builtin_amdgcn_s_sleep(1);
        }
        if (!ok && lane == 0) {
          give_up = 1;
          __hip_atomic_store(a.status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
      __syncthreads();
      if (give_up) break;
    }
    const T *hblk = static_cast<const T *>(a.Hs) + (int64_t)t * a.B * a.h_pitch;
    floatx16 acc0, acc1;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc0[v] = acc1[v] = 0.0f;
    copy_h(stage0, hblk, 0);
    if (n_chunks > 1) copy_h(stage1, hblk, 1);
    auto step = [&](char *cur, int ch) {
      // the copies of chunk ch are older than those of chunk ch + 1, which may stay in flight (8 per wave and chunk)
      if (ch + 1 < n_chunks) __builtin_amdgcn_s_waitcnt(0x0F78); else __builtin_amdgcn_s_waitcnt(0x0F70);
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      mma_chunk(acc0, acc1, cur, ch);
      __builtin_amdgcn_s_waitcnt(0xC07F);         // lgkmcnt(0): the fragment reads have returned
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      if (ch + 2 < n_chunks) copy_h(cur, hblk, ch + 2);
    };
#pragma unroll 1
    for (int ch = 0; ch < n_chunks; ch += 2) {
      step(stage0, ch);
      if (ch + 1 < n_chunks) step(stage1, ch + 1);
    }
    // ---- partial tiles meet in LDS; the cell
    {
      const int r = lane & 31, q = lane >> 5;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        tile0[wave][8 * (v / 4) + 4 * q + v % 4][r] = acc0[v];
        tile1[wave][8 * (v / 4) + 4 * q + v % 4][r] = acc1[v];
      }
    }
    __syncthreads();
    if (live) {
      float (*tile)[32][33] = crow < 32 ? tile0 : tile1;
      const int tr = crow & 31;
      float hv[2], gate[4][2];
#pragma unroll
      for (int e = 0; e < 2; ++e) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int col = 8 * g + jj + e;
          z[g][e] += (tile[0][tr][col] + tile[1][tr][col]) + (tile[2][tr][col] + tile[3][tr][col]);
        }
        const float i = sigmoid_f(z[0][e]), f = sigmoid_f(z[1][e]), g = tanhf(z[2][e]), o = sigmoid_f(z[3][e]);
        c_state[e] = f * c_state[e] + i * g;
        hv[e] = o * tanhf(c_state[e]);
        gate[0][e] = i; gate[1][e] = f; gate[2][e] = g; gate[3][e] = o;
      }
      const int64_t out_row = (int64_t)(t + 1) * a.B + b;
      store_h2(static_cast<T *>(a.Hs) + out_row * a.h_pitch + j, hv[0], hv[1]);
      float *cr = a.Cs + out_row * a.c_pitch + j;
      cr[0] = c_state[0]; cr[1] = c_state[1];
      if (a.gates) {
        float *gr = a.gates + ((int64_t)t * a.B + b) * a.g_pitch;
#pragma unroll
        for (int g = 0; g < 4; ++g) { gr[g * a.H + j] = gate[g][0]; gr[g * a.H + j + 1] = gate[g][1]; }
      }
    }
    // ---- publish: every thread's stores are done, then one arrival for the workgroup
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    if (threadIdx.x == 0 && t + 1 < a.n_steps)
      __hip_atomic_fetch_add(a.counters + blockIdx.y, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

std::atomic<int> g_spin_limit{1 << 20};

chn_status view2(const chn_array *x, const char *name, bool out, int64_t rows, int64_t cols, int want_dtype, bool operand, int64_t *pitch) {
  CHN_TRY(validate(x, name, out));
  if (x->dtype != want_dtype) return fail(CHN_ERR_DTYPE, "lstm_seq: %s must be %s", name, want_dtype == CHN_F32 ? "F32" : "BF16");
  int64_t r, c;
  CHN_TRY(row_major_2d(x, name, &r, &c, pitch));
  if (r != rows || c != cols) return fail(CHN_ERR_SHAPE, "lstm_seq: %s must have shape (%lld,%lld)", name, (long long)rows, (long long)cols);
  if (operand) {
    const int per16 = 16 / dtype_size(x->dtype);
    if (reinterpret_cast<uintptr_t>(x->data) % 16 || (rows > 1 && *pitch % per16))
      return fail(CHN_ERR_STRIDE, "lstm_seq: rows of %s must start on 16-byte boundaries", name);
  }
  return CHN_OK;
}

// What the resident grid can hold: the slice of Ut in LDS, every workgroup on a compute unit of its own.
chn_status fits(int64_t B, int64_t H, int dtype) {
  if (dtype != CHN_F32 && dtype != CHN_BF16) return fail(CHN_ERR_DTYPE, "lstm_seq: h and Ut must be F32 or BF16");
  const int isz = (int)dtype_size(dtype);
  if (B < 0 || H < 0) return fail(CHN_ERR_SHAPE, "lstm_seq: negative extent");
  if (H % (32 / isz)) return fail(CHN_ERR_SHAPE, "lstm_seq: the hidden width %lld is not a multiple of %d", (long long)H, 32 / isz);
  if (H * isz > (int64_t)kMaxChunks * kRowBytes)
    return fail(CHN_ERR_SHAPE, "lstm_seq: a row of h has %lld bytes, the resident slice of Ut holds rows of up to %d (use the per-step calls)",
                (long long)(H * isz), kMaxChunks * kRowBytes);
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
    return fail(CHN_ERR_LAUNCH, "lstm_seq: cannot ask the device for its number of compute units");
  const int64_t need = ((B + 63) / 64) * (H / 8);
  if (need > cus)
    return fail(CHN_ERR_SHAPE, "lstm_seq: %lld workgroups needed, the device has %d compute units (use the per-step calls)", (long long)need, cus);
  return CHN_OK;
}

}  // namespace
}  // namespace chn

extern "C" {

chn_status chn_lstm_seq_supported(int64_t batch, int64_t hidden, int dtype) { return chn::fits(batch, hidden, dtype); }

size_t chn_lstm_seq_workspace_bytes(int64_t batch) {
  if (batch <= 0) return 0;
  return 256 + (size_t)((batch + 63) / 64) * sizeof(unsigned) + 256;
}

void chn_lstm_seq_spin_limit(int64_t polls) { chn::g_spin_limit.store(polls < 0 ? 0 : polls > (1 << 30) ? (1 << 30) : (int)polls); }

chn_status chn_lstm_seq_fwd(const chn_array *zx, const chn_array *Ut, const chn_array *bias, const chn_array *Hs, const chn_array *Cs,
                            const chn_array *gates, int64_t n_steps, void *ws, size_t ws_bytes, chn_stream stream) {
  using namespace chn;
  CHN_TRY(validate(Cs, "Cs", true));
  if (Cs->ndim != 2) return fail(CHN_ERR_NDIM, "lstm_seq: Cs must be 2-d");
  if (!Hs || !Ut) return fail(CHN_ERR_NULL, "lstm_seq: Hs or Ut is NULL");
  if (n_steps < 0 || n_steps > (1 << 20)) return fail(CHN_ERR_SHAPE, "lstm_seq: bad number of steps %lld", (long long)n_steps);
  SeqArgs a{};
  a.H = Cs->shape[1];
  const int64_t rows = Cs->shape[0];
  if (rows % (n_steps + 1)) return fail(CHN_ERR_SHAPE, "lstm_seq: Cs has %lld rows, not a multiple of steps + 1 = %lld", (long long)rows, (long long)(n_steps + 1));
  a.B = rows / (n_steps + 1);
  const int t = Hs->dtype;
  CHN_TRY(fits(a.B, a.H, t));
  CHN_TRY(view2(Cs, "Cs", true, rows, a.H, CHN_F32, false, &a.c_pitch));
  CHN_TRY(view2(Hs, "Hs", true, rows, a.H, t, true, &a.h_pitch));
  CHN_TRY(view2(zx, "zx", false, n_steps * a.B, 4 * a.H, CHN_F32, false, &a.zx_pitch));
  CHN_TRY(view2(Ut, "Ut", false, 4 * a.H, a.H, t, true, &a.ut_pitch));
  if (gates) CHN_TRY(view2(gates, "gates", true, n_steps * a.B, 4 * a.H, CHN_F32, false, &a.g_pitch));
  if (bias) {
    CHN_TRY(validate(bias, "bias", false));
    if (bias->dtype != CHN_F32 || bias->ndim != 1 || bias->shape[0] != 4 * a.H || !is_contiguous(bias))
      return fail(CHN_ERR_SHAPE, "lstm_seq: bias must be a contiguous F32 (%lld,) array", (long long)(4 * a.H));
  }
  if (n_steps == 0 || a.B * a.H == 0) return CHN_OK;
  // 8-byte (F32) / 4-byte (BF16) stores of two neighbouring units: rows of h on such boundaries
  if ((a.h_pitch * dtype_size(t)) % 8 && t == CHN_F32) return fail(CHN_ERR_STRIDE, "lstm_seq: rows of Hs must start on 8-byte boundaries");
  const int64_t nbb = (a.B + 63) / 64, nub = a.H / 8;
  CHN_TRY(check_ws(ws, ws_bytes, chn_lstm_seq_workspace_bytes(a.B), "lstm_seq"));
  a.n_steps = (int)n_steps; a.nub = (int)nub; a.spin_limit = g_spin_limit.load();
  a.zx = static_cast<const float *>(zx->data);
  a.Ut = Ut->data;
  a.bias = bias ? static_cast<const float *>(bias->data) : nullptr;
  a.Hs = Hs->data;
  a.Cs = static_cast<float *>(Cs->data);
  a.gates = gates ? static_cast<float *>(gates->data) : nullptr;
  a.status = static_cast<unsigned *>(ws);
  a.counters = reinterpret_cast<unsigned *>(static_cast<char *>(ws) + 256);
  hipStream_t st = as_stream(stream);
  hipLaunchKernelGGL(seq_clear_kernel, dim3(1), dim3(64), 0, st, a.status, (int)(64 + nbb));
  CHN_TRY(check_launch("lstm_seq clear"));
  const dim3 grid((unsigned)nub, (unsigned)nbb);
  if (t == CHN_BF16) hipLaunchKernelGGL(lstm_seq_fwd_kernel<bf16_raw>, grid, dim3(kThreads), 0, st, a);
  else hipLaunchKernelGGL(lstm_seq_fwd_kernel<float>, grid, dim3(kThreads), 0, st, a);
  return check_launch("lstm_seq_fwd");
}

}  // extern "C"
