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
#include <type_traits>

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

// two row blocks against the same piece of the other operand, the two accumulator chains taking turns
template <typename T>
__device__ __forceinline__ void mma_pair(floatx16 &acc0, floatx16 &acc1, const uint4 &a0, const uint4 &a1, const uint4 &b) {
  if constexpr (sizeof(T) == 2) {
    mma_piece<T>(acc0, a0, b);
    mma_piece<T>(acc1, a1, b);
  } else {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float((&a0.x)[kk]), __uint_as_float((&b.x)[kk]), acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float((&a1.x)[kk]), __uint_as_float((&b.x)[kk]), acc1, 0, 0, 0);
    }
  }
}

// Activations of the cell on the hardware's exponential and reciprocal (relative error a few 1e-7): between two
// exchanges the cell is on the critical path of every step, and the library's expf / tanhf are a third of it.
__device__ __forceinline__ float sigmoid_hw(float x) { return __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }
// tanh: (1 - e) / (1 + e) with e = exp(-2 |x|) cancels for small |x|; there the odd series takes over (its first
// dropped term, 62/2835 x^9, is below 1e-7 of x for |x| < 0.25), so that the relative error stays at a few 1e-7.
__device__ __forceinline__ float tanh_hw(float x) {
  const float ax = fabsf(x), e = __expf(-2.0f * ax);
  const float big = copysignf((1.0f - e) * __builtin_amdgcn_rcpf(1.0f + e), x);
  const float x2 = x * x;
  const float small = x * fmaf(x2, fmaf(x2, fmaf(x2, -17.0f / 315.0f, 2.0f / 15.0f), -1.0f / 3.0f), 1.0f);
  return ax < 0.25f ? small : big;
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
// UC: 512-byte chunks of a row of Ut the resident slice holds; NS: stages the rows of h stream through.  What the
// slice leaves free of the 160 KB goes to stages: with rows of three chunks (H <= 384 F32, 768 BF16) all of h_{t-1}
// is in flight at once and a step pays the latency of device memory once instead of once per chunk.
template <typename T, int UC, int NS>
__global__ __launch_bounds__(kThreads) void lstm_seq_fwd_kernel(SeqArgs a) {
  static_assert(UC * kUChunkBytes + NS * kHStageBytes <= 160 * 1024 && NS >= 2 && NS <= 4, "LDS budget");
  __shared__ __attribute__((aligned(1024))) char uslice[UC * kUChunkBytes];
  __shared__ __attribute__((aligned(1024))) char stage0[kHStageBytes];
  __shared__ __attribute__((aligned(1024))) char stage1[kHStageBytes];
  __shared__ __attribute__((aligned(1024))) char stage2_[kHStageBytes];     // allocated only where referenced
  __shared__ __attribute__((aligned(1024))) char stage3_[kHStageBytes];
  char *stage2 = stage0, *stage3 = stage0;
  if constexpr (NS > 2) stage2 = stage2_;
  if constexpr (NS > 3) stage3 = stage3_;
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
  // A wave's share of a staged chunk: every fourth 32-byte slice (slices 4 u + wave: the slices of a partial last chunk
  // are dealt out over the waves too), against the resident rows of Ut.  The fragments of chunk c + 1 are read while
  // the matrix cores work on chunk c, into the other of two register sets.
  struct Frag { uint4 x0[4], x1[4], y[4]; };
  auto slices_of = [&](int ch) {
    const int64_t left = row_bytes - (int64_t)ch * kRowBytes;
    return (int)((left < kRowBytes ? left : kRowBytes) / 32);
  };
  auto read_frags = [&](Frag &f, const char *stage, int ch) __attribute__((always_inline)) {
    const int n_slices = slices_of(ch);
    const int r = lane & 31, q = lane >> 5;
    const char *pa = stage + r * kRowBytes, *pb = uslice + ch * kUChunkBytes + r * kRowBytes;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int s = 4 * u + wave;
      if (s < n_slices) {
        const int pos = ((2 * s + q) ^ (r & 15)) << 4;
        f.x0[u] = *reinterpret_cast<const uint4 *>(pa + pos);
        f.x1[u] = *reinterpret_cast<const uint4 *>(pa + 32 * kRowBytes + pos);
        f.y[u] = *reinterpret_cast<const uint4 *>(pb + pos);
      }
    }
  };
  auto mma_frags = [&](floatx16 &acc0, floatx16 &acc1, const Frag &f, int ch) __attribute__((always_inline)) {
    const int n_slices = slices_of(ch);
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (4 * u + wave < n_slices) mma_pair<T>(acc0, acc1, f.x0[u], f.x1[u], f.y[u]);
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
    if (NS > 2 && n_chunks > 2) copy_h(stage2, hblk, 2);
    if (NS > 3 && n_chunks > 3) copy_h(stage3, hblk, 3);
    // the copies of a chunk are older than those of the chunks after it, which may stay in flight (8 per wave and chunk)
    auto wait_copies = [&](int newer) __attribute__((always_inline)) {
      if (newer <= 0) __builtin_amdgcn_s_waitcnt(0x0F70);
      else if (newer == 1) __builtin_amdgcn_s_waitcnt(0x0F78);
      else if (newer == 2) __builtin_amdgcn_s_waitcnt(0x4F70);       // vmcnt(16)
      else __builtin_amdgcn_s_waitcnt(0x4F78);                       // vmcnt(24)
    };
    auto barrier = [&]() __attribute__((always_inline)) {
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
    };
    char *const stages[4] = {stage0, stage1, stage2, stage3};
    Frag fa, fb;
    wait_copies(n_chunks - 1 < NS - 1 ? n_chunks - 1 : NS - 1);
    barrier();
    read_frags(fa, stage0, 0);
    // Chunk by chunk (at most kMaxChunks; written out so that stage and register set are named at compile time):
    // the fragments of chunk ch have been requested.  Once they are here and the copies of chunk ch + 1 have landed,
    // one barrier says both for every wave: the stage of chunk ch may be refilled and chunk ch + 1 may be read -
    // which then happens under the MFMAs of chunk ch.
#pragma unroll
    for (int ch = 0; ch < kMaxChunks; ++ch) {
      if (ch < n_chunks) {
        Frag &cur = ch % 2 ? fb : fa, &nxt = ch % 2 ? fa : fb;
        if (ch + 1 < n_chunks) {
          __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0): this wave's fragment reads of chunk ch are back
          wait_copies(n_chunks - 2 - ch < NS - 2 ? n_chunks - 2 - ch : NS - 2);
          barrier();
          if (ch + NS < n_chunks) copy_h(stages[ch % NS], hblk, ch + NS);
          read_frags(nxt, stages[(ch + 1) % NS], ch + 1);
        }
        mma_frags(acc0, acc1, cur, ch);
      }
    }
    // every wave is done with the stages before the partial tiles overwrite them
    barrier();
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
        const float i = sigmoid_hw(z[0][e]), f = sigmoid_hw(z[1][e]), g = tanh_hw(z[2][e]), o = sigmoid_hw(z[3][e]);
        c_state[e] = f * c_state[e] + i * g;
        hv[e] = o * tanh_hw(c_state[e]);
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

// ------------------------------------------------------------------------------------------------------------
// Back-propagation through time in one launch.  dh_t = (gradient from above) + dz_{t+1} U^T is a contraction over
// the 4H gate columns; cut along THAT axis, a workgroup that owns 16 hidden units (64 gate columns) for 32 batch
// rows multiplies the dz it has just produced itself - no operand to fetch - with its 64 columns of U, which it
// keeps in REGISTERS for the whole sequence (the matrix cores take them from there: nothing of U is read again
// after the first step, not even from LDS).  What comes out is a partial dh for all H units; the H / 16
// workgroups of a batch block exchange those through device memory (each writes one 2 KB block per receiver,
// each receiver reads its H / 16 blocks back to back and adds them in a fixed order) with the same agent-scope
// stores, arrival counter and bounded wait as the forward kernel, then run the cell's backward on their own units.
struct SeqBwdArgs {
  int64_t B, H;
  int n_steps, nub, spin_limit;
  const void *U; int64_t u_pitch;
  void *dHs; int64_t dh_pitch;
  const float *gates; int64_t g_pitch;
  const float *Cs; int64_t c_pitch;
  const float *dc_last; int64_t dcl_pitch;
  void *dZ; int64_t dz_pitch;
  float *dc0; int64_t dc0_pitch;
  float *xbuf;               // [2][batch blocks][receiver][sender][2][32 rows][8 units]
  unsigned *counters, *status;
};

constexpr int kBwdRows = 32, kBwdUnits = 16, kBwdCols = 4 * kBwdUnits;
constexpr int kBlockFloats = kBwdRows * kBwdUnits;     // one sender -> receiver block
constexpr int kBatchLoads = 48;                        // blocks a thread has in flight at once

// grid: (H / 16, ceil(B / 32)).  MT: the most 32-unit row tiles of U a wave holds (tiles wave, wave + 4, ...).
template <typename T, int MT>
__global__ __launch_bounds__(kThreads) void lstm_seq_bwd_kernel(SeqBwdArgs a) {
  constexpr int NI = sizeof(T) == 2 ? 4 : 8;           // 16-byte pieces along the 64 gate columns per lane half
  constexpr int kTileRow = kBwdCols * (int)sizeof(T);  // bytes of one row of the dz tile
  constexpr int kSwz = kTileRow / 16 - 1;
  __shared__ __attribute__((aligned(16))) char tile[kBwdRows * kTileRow];
  __shared__ int give_up;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  const int r = lane & 31, q = lane >> 5;
  const int64_t j0 = (int64_t)blockIdx.x * kBwdUnits, b0 = (int64_t)blockIdx.y * kBwdRows;
  const int n_mt = (int)((a.H + 31) / 32);
  const int T_ = a.n_steps;

  // ---- this wave's rows of U (all H units, this workgroup's 64 gate columns), once, into registers
  uint4 ua[MT][NI];
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    const int mt = wave + 4 * m;
    int64_t row = (int64_t)mt * 32 + r;
    if (row >= a.H) row = a.H - 1;
    const T *ur = static_cast<const T *>(a.U) + row * a.u_pitch;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      // piece i of lane half q covers gate columns c = (16 / sizeof(T)) * (2 i + q) ..: gate c / 16, unit c % 16
      const int c = (16 / (int)sizeof(T)) * (2 * i + q);
      ua[m][i] = *reinterpret_cast<const uint4 *>(ur + (int64_t)(c >> 4) * a.H + j0 + (c & 15));   // tiles past the last repeat its last row; never used
    }
  }
  // nothing of this is in flight when the step loop starts: no wait on these registers inside it
  __builtin_amdgcn_s_waitcnt(0x0F70);
  asm volatile("" ::: "memory");

  // ---- this thread's part of the cell: one batch row, two neighbouring hidden units
  const int crow = threadIdx.x >> 3, cp2 = threadIdx.x & 7;
  const int64_t b = b0 + crow, j = j0 + 2 * cp2;
  const bool live = b < a.B;
  float dc[2] = {0.0f, 0.0f};
  if (live && a.dc_last) { dc[0] = a.dc_last[b * a.dcl_pitch + j]; dc[1] = a.dc_last[b * a.dcl_pitch + j + 1]; }
  const int64_t blocks_per_bb = (int64_t)a.nub * a.nub;
  // the exchange buffer as a buffer resource: stores carry a cache policy and are range-checked by the hardware
  const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(a.xbuf, 0, (int)(2 * gridDim.y * blocks_per_bb * kBlockFloats * 4), 0x00020000);
  if (threadIdx.x == 0) give_up = 0;

#pragma unroll 1
  for (int step = 0; step < T_; ++step) {
    const int t = T_ - 1 - step;
    // what the cell's backward reads, fetched before the exchange
    // (raw bits: nothing here is looked at before the exchange is over, so nothing waits for it earlier)
    float gt[4][2], cc[2], cprev[2], d[2];
    typedef typename std::conditional<sizeof(T) == 2, unsigned, float2>::type Pair;
    Pair d_raw{};
#pragma unroll
    for (int e = 0; e < 2; ++e) { cc[e] = cprev[e] = 0.0f; gt[0][e] = gt[1][e] = gt[2][e] = gt[3][e] = 0.0f; }
    T *dhr = static_cast<T *>(a.dHs) + ((int64_t)t * a.B + b) * a.dh_pitch + j;
    if (live) {
      const float *gr = a.gates + ((int64_t)t * a.B + b) * a.g_pitch;
      const float *cr = a.Cs + ((int64_t)(t + 1) * a.B + b) * a.c_pitch + j, *pr = a.Cs + ((int64_t)t * a.B + b) * a.c_pitch + j;
#pragma unroll
      for (int e = 0; e < 2; ++e) {
#pragma unroll
        for (int g = 0; g < 4; ++g) gt[g][e] = gr[g * a.H + j + e];
        cc[e] = cr[e]; cprev[e] = pr[e];
      }
      d_raw = *reinterpret_cast<const Pair *>(dhr);
    }
    d[0] = d[1] = 0.0f;
    if (step > 0) {
      const int xoff = (int)(((int64_t)(step & 1) * gridDim.y + blockIdx.y) * blocks_per_bb * kBlockFloats * 4);   // bytes; the exchange stays under 2 GiB
      const float *xb = a.xbuf + xoff / 4;
      // ---- partial dh of all units from this workgroup's dz of step t + 1 (in the LDS tile)
      uint4 bf[NI];
#pragma unroll
      for (int i = 0; i < NI; ++i) bf[i] = *reinterpret_cast<const uint4 *>(tile + r * kTileRow + (((2 * i + q) ^ (r & kSwz)) << 4));
#pragma unroll
      for (int m = 0; m < MT; ++m) {
        const int mt = wave + 4 * m;
        if (mt < n_mt) {
          floatx16 acc;
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
          for (int i = 0; i < NI; ++i) mma_piece<T>(acc, ua[m][i], bf[i]);
          // rows of the result = units 32 mt + 8 (v / 4) + 4 q + v % 4, columns = batch rows r
#pragma unroll
          for (int vg = 0; vg < 4; ++vg) {
            const int dest = 2 * mt + (vg >> 1);
            if (dest < a.nub) {
              // 16 bytes per lane, 1 KB back to back per instruction, written through to device memory (sc0 sc1)
              const int off = xoff + (dest * a.nub + (int)blockIdx.x) * (kBlockFloats * 4) + (vg & 1) * (kBwdRows * 32) + r * 32 + q * 16;
              const chn_f32x4 val = {acc[4 * vg], acc[4 * vg + 1], acc[4 * vg + 2], acc[4 * vg + 3]};
              __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(chn_u32x4, val), xres, off, 0, kCpolAgent);
            }
          }
        }
      }
      // ---- publish, then wait for the other workgroups of this batch block
      __builtin_amdgcn_s_waitcnt(0x0F70);
      __syncthreads();
      if (threadIdx.x == 0) __hip_atomic_fetch_add(a.counters + blockIdx.y, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (wave == 0) {
        const unsigned want = (unsigned)step * (unsigned)a.nub;
        bool ok = false;
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
      // ---- the partial sums addressed to this workgroup, one block per sender, added in sender order
      const float *mine = xb + (int64_t)blockIdx.x * a.nub * kBlockFloats + (cp2 >> 2) * (kBwdRows * 8) + crow * 8 + 2 * (cp2 & 3);
      float rec0 = 0.0f, rec1 = 0.0f;
#pragma unroll 1
      for (int s0 = 0; s0 < a.nub; s0 += kBatchLoads) {
        unsigned long long v[kBatchLoads];
#pragma unroll
        for (int s = 0; s < kBatchLoads; ++s)
          v[s] = s0 + s < a.nub ? __hip_atomic_load(reinterpret_cast<const unsigned long long *>(mine + (int64_t)(s0 + s) * kBlockFloats),
                                                    __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                : 0ull;
#pragma unroll
        for (int s = 0; s < kBatchLoads; ++s) {
          rec0 += __uint_as_float((unsigned)v[s]);
          rec1 += __uint_as_float((unsigned)(v[s] >> 32));
        }
      }
      d[0] = rec0; d[1] = rec1;
    }
    if constexpr (sizeof(T) == 2) { d[0] += bf16_to_f32((bf16_raw)(d_raw & 0xFFFFu)); d[1] += bf16_to_f32((bf16_raw)(d_raw >> 16)); }
    else { d[0] += d_raw.x; d[1] += d_raw.y; }
    if (step > 0) {
      // the total is what the cell sees and what is stored: in mixed precision that is the bf16 value
      if (live) { Elem<T>::store(dhr, d[0]); Elem<T>::store(dhr + 1, d[1]); }
      if constexpr (sizeof(T) == 2) { d[0] = bf16_to_f32(f32_to_bf16(d[0])); d[1] = bf16_to_f32(f32_to_bf16(d[1])); }
    }
    // ---- the cell's backward; dz goes to memory and, as the operand of the next step's product, into the tile
    float dzv[4][2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const float i = gt[0][e], f = gt[1][e], g = gt[2][e], o = gt[3][e];
      const float tc = tanhf(cc[e]);
      const float d_o = d[e] * tc;
      const float dcv = dc[e] + d[e] * o * (1.0f - tc * tc);
      const float di = dcv * g, dg = dcv * i, df = dcv * cprev[e];
      dc[e] = dcv * f;
      dzv[0][e] = di * i * (1.0f - i);
      dzv[1][e] = df * f * (1.0f - f);
      dzv[2][e] = dg * (1.0f - g * g);
      dzv[3][e] = d_o * o * (1.0f - o);
    }
    T *dzr = static_cast<T *>(a.dZ) + ((int64_t)t * a.B + b) * a.dz_pitch + j;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int c = g * kBwdUnits + 2 * cp2;               // column of the tile; c and c + 1 share a 16-byte piece
      constexpr int per = 16 / (int)sizeof(T);
      char *pt = tile + crow * kTileRow + (((c / per) ^ (crow & kSwz)) << 4) + (c % per) * (int)sizeof(T);
      if constexpr (sizeof(T) == 2) {
        const unsigned bits = live ? (unsigned)f32_to_bf16(dzv[g][0]) | ((unsigned)f32_to_bf16(dzv[g][1]) << 16) : 0u;
        *reinterpret_cast<unsigned *>(pt) = bits;
        if (live) *reinterpret_cast<unsigned *>(dzr + g * a.H) = bits;
      } else {
        const float2 v = live ? float2{dzv[g][0], dzv[g][1]} : float2{0.0f, 0.0f};
        *reinterpret_cast<float2 *>(pt) = v;
        if (live) *reinterpret_cast<float2 *>(dzr + g * a.H) = v;
      }
    }
    __syncthreads();
  }
  if (live && !give_up) { a.dc0[b * a.dc0_pitch + j] = dc[0]; a.dc0[b * a.dc0_pitch + j + 1] = dc[1]; }
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

// What the backward grid can hold: the tiles of U in registers, every workgroup resident.
chn_status fits_bwd(int64_t B, int64_t H, int dtype) {
  if (dtype != CHN_F32 && dtype != CHN_BF16) return fail(CHN_ERR_DTYPE, "lstm_seq_bwd: U and the gradients must be F32 or BF16");
  if (B < 0 || H < 0) return fail(CHN_ERR_SHAPE, "lstm_seq_bwd: negative extent");
  if (H % kBwdUnits) return fail(CHN_ERR_SHAPE, "lstm_seq_bwd: the hidden width %lld is not a multiple of %d", (long long)H, kBwdUnits);
  const int64_t widest = dtype == CHN_F32 ? 768 : 1536;
  if (H > widest)
    return fail(CHN_ERR_SHAPE, "lstm_seq_bwd: hidden width %lld; the registers hold the rows of U up to %lld (use the per-step calls)", (long long)H, (long long)widest);
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
    return fail(CHN_ERR_LAUNCH, "lstm_seq_bwd: cannot ask the device for its number of compute units");
  const int64_t need = ((B + kBwdRows - 1) / kBwdRows) * (H / kBwdUnits);
  if (need > cus)
    return fail(CHN_ERR_SHAPE, "lstm_seq_bwd: %lld workgroups needed, the device has %d compute units (use the per-step calls)", (long long)need, cus);
  return CHN_OK;
}

size_t bwd_exchange_bytes(int64_t B, int64_t H) {
  const int64_t nbb = (B + kBwdRows - 1) / kBwdRows, nub = H / kBwdUnits;
  return (size_t)(2 * nbb * nub * nub) * kBlockFloats * sizeof(float);
}
size_t bwd_counter_bytes(int64_t B) { return (size_t)((((B + kBwdRows - 1) / kBwdRows) * sizeof(unsigned) + 255) / 256 * 256); }

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
  const int64_t chunks = (a.H * dtype_size(t) + kRowBytes - 1) / kRowBytes;
#define CHN_SEQ_FWD(UC, NS)                                                                                            \
  do {                                                                                                                 \
    if (t == CHN_BF16) hipLaunchKernelGGL((lstm_seq_fwd_kernel<bf16_raw, UC, NS>), grid, dim3(kThreads), 0, st, a);    \
    else hipLaunchKernelGGL((lstm_seq_fwd_kernel<float, UC, NS>), grid, dim3(kThreads), 0, st, a);                     \
  } while (0)
  if (chunks <= 2) CHN_SEQ_FWD(2, 4);
  else if (chunks <= 3) CHN_SEQ_FWD(3, 3);
  else if (chunks <= 4) CHN_SEQ_FWD(4, 3);
  else CHN_SEQ_FWD(6, 2);
#undef CHN_SEQ_FWD
  return check_launch("lstm_seq_fwd");
}

chn_status chn_lstm_seq_bwd_supported(int64_t batch, int64_t hidden, int dtype) { return chn::fits_bwd(batch, hidden, dtype); }

size_t chn_lstm_seq_bwd_workspace_bytes(int64_t batch, int64_t hidden) {
  if (batch <= 0 || hidden <= 0 || hidden % chn::kBwdUnits) return 0;
  return 256 + chn::bwd_counter_bytes(batch) + chn::bwd_exchange_bytes(batch, hidden);
}

chn_status chn_lstm_seq_bwd(const chn_array *U, const chn_array *dHs, const chn_array *gates, const chn_array *Cs,
                            const chn_array *dc_last, const chn_array *dZ, const chn_array *dc0, int64_t n_steps, void *ws,
                            size_t ws_bytes, chn_stream stream) {
  using namespace chn;
  CHN_TRY(validate(Cs, "Cs", false));
  if (Cs->ndim != 2) return fail(CHN_ERR_NDIM, "lstm_seq_bwd: Cs must be 2-d");
  if (!U || !dHs || !dZ) return fail(CHN_ERR_NULL, "lstm_seq_bwd: U, dHs or dZ is NULL");
  if (n_steps < 0 || n_steps > (1 << 20)) return fail(CHN_ERR_SHAPE, "lstm_seq_bwd: bad number of steps %lld", (long long)n_steps);
  SeqBwdArgs a{};
  a.H = Cs->shape[1];
  const int64_t rows = Cs->shape[0];
  if (rows % (n_steps + 1)) return fail(CHN_ERR_SHAPE, "lstm_seq_bwd: Cs has %lld rows, not a multiple of steps + 1 = %lld", (long long)rows, (long long)(n_steps + 1));
  a.B = rows / (n_steps + 1);
  const int t = U->dtype;
  CHN_TRY(fits_bwd(a.B, a.H, t));
  const int64_t n = n_steps * a.B;
  CHN_TRY(view2(Cs, "Cs", false, rows, a.H, CHN_F32, false, &a.c_pitch));
  CHN_TRY(view2(U, "U", false, a.H, 4 * a.H, t, true, &a.u_pitch));
  CHN_TRY(view2(dHs, "dHs", true, n, a.H, t, false, &a.dh_pitch));
  CHN_TRY(view2(gates, "gates", false, n, 4 * a.H, CHN_F32, false, &a.g_pitch));
  CHN_TRY(view2(dZ, "dZ", true, n, 4 * a.H, t, false, &a.dz_pitch));
  CHN_TRY(view2(dc0, "dc0", true, a.B, a.H, CHN_F32, false, &a.dc0_pitch));
  if (dc_last) CHN_TRY(view2(dc_last, "dc_last", false, a.B, a.H, CHN_F32, false, &a.dcl_pitch));
  if (n_steps == 0 || a.B * a.H == 0) return CHN_OK;
  // dz leaves in pairs of neighbouring units (8 bytes F32, 4 bytes BF16)
  if (reinterpret_cast<uintptr_t>(dZ->data) % 8 || (a.dz_pitch * dtype_size(t)) % 8)
    return fail(CHN_ERR_STRIDE, "lstm_seq_bwd: rows of dZ must start on 8-byte boundaries");
  const size_t need = chn_lstm_seq_bwd_workspace_bytes(a.B, a.H);
  CHN_TRY(check_ws(ws, ws_bytes, need, "lstm_seq_bwd"));
  const int64_t nbb = (a.B + kBwdRows - 1) / kBwdRows, nub = a.H / kBwdUnits;
  a.n_steps = (int)n_steps; a.nub = (int)nub; a.spin_limit = g_spin_limit.load();
  a.U = U->data;
  a.dHs = dHs->data;
  a.gates = static_cast<const float *>(gates->data);
  a.Cs = static_cast<const float *>(Cs->data);
  a.dc_last = dc_last ? static_cast<const float *>(dc_last->data) : nullptr;
  a.dZ = dZ->data;
  a.dc0 = static_cast<float *>(dc0->data);
  a.status = static_cast<unsigned *>(ws);
  a.counters = reinterpret_cast<unsigned *>(static_cast<char *>(ws) + 256);
  a.xbuf = reinterpret_cast<float *>(static_cast<char *>(ws) + 256 + bwd_counter_bytes(a.B));
  hipStream_t st = as_stream(stream);
  hipLaunchKernelGGL(seq_clear_kernel, dim3(1), dim3(64), 0, st, a.status, (int)(64 + nbb));
  CHN_TRY(check_launch("lstm_seq_bwd clear"));
  const dim3 grid((unsigned)nub, (unsigned)nbb);
  if (t == CHN_BF16) hipLaunchKernelGGL((lstm_seq_bwd_kernel<bf16_raw, 12>), grid, dim3(kThreads), 0, st, a);
  else hipLaunchKernelGGL((lstm_seq_bwd_kernel<float, 6>), grid, dim3(kThreads), 0, st, a);
  return check_launch("lstm_seq_bwd");
}

}  // extern "C"
