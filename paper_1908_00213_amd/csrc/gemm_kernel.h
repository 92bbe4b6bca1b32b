// chn_gemm: C = epilogue(alpha * A B + beta * C) on the gfx950 matrix cores.
//
// The paper's fully connected layer (figure "Examples of model definitions": y = x @ W.T + b) and its
// two backward products are the one dense contraction of a training step, so this is the one place
// that uses MFMA: v_mfma_f32_32x32x16_bf16 for bfloat16 operands and v_mfma_f32_32x32x2_f32 for fp32
// operands, always accumulating in fp32.
//
// Structure of one workgroup (256 threads = 4 waves in a 2x2 arrangement):
//   * macro tile (64*TM) x (64*TN) of C, TM = TN in {4, 2, 1}; each wave owns TM x TN MFMA blocks
//     of 32x32, i.e. up to 128x128 accumulators per wave held in registers;
//   * the K loop advances one "tile step" of 128 bytes of K per operand row (64 bf16 or 32 fp32),
//     made of four "k-steps" of two 16-byte chunks.  Operand tiles live in LDS as rows of 128 bytes
//     = 8 chunks of 16 bytes, always K-packed, with the chunk index XOR-swizzled by (row/2)%8 so that
//     neither the 16-byte stores nor the 16-byte MFMA fragment reads collide on LDS banks, without
//     padding; two such stages (double buffering);
//   * operands whose unit stride runs along K are copied chunk by chunk; operands whose unit stride
//     runs along M/N (transposed views) are loaded in 16-byte pieces along M/N and transposed in
//     registers (8x8 bf16 or 4x4 fp32 blocks) on their way into LDS, so the inner loop is the same
//     for all four layout combinations and no second copy of an operand is ever made;
//   * software pipeline of one tile step (one wave per SIMD has nobody to hide its latencies, so the
//     order is explicit): k-steps 0..2 multiply out of the current stage while the fragments of the
//     following k-step are already being read; k-step 0 also issues the global loads of the next
//     tile into registers, k-step 2 writes them to the other stage; one barrier; k-step 3 multiplies
//     while the first fragments of the next stage are read;
//   * since the sum over k is order-free, the 16 (8) k-values one lane feeds to an MFMA need not be
//     the hardware's nominal ones as long as A and B agree; each lane therefore reads one whole
//     16-byte chunk per 32 rows and k-step;
//   * workgroups are renumbered so that the eight XCDs (which take consecutive workgroup ids
//     round-robin) each work on a compact patch of C tiles and share operand tiles in their own L2;
//   * the epilogue stages each wave's accumulators through LDS (the operand stages are free by then)
//     so that bias / activation / activation-gradient run on 16-byte vectors and C, aux and preact
//     are accessed as whole 512-byte (fp32) or 256-byte (bf16) row segments; one final rounding.
#pragma once
#include <type_traits>

#include "common.h"
#include "gemm_args.h"

namespace chn {
namespace gemm {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <typename T> struct Traits;
template <> struct Traits<float> { static constexpr int EPC = 4; };      // elements per 16-byte chunk
template <> struct Traits<bf16_raw> { static constexpr int EPC = 8; };

// Byte offset of logical chunk q of tile row `row` inside a stage.  Two swizzles: the chunk index is
// XORed with (row/2)%8, and rows swap places pairwise (row ^ 1) when bit log2(EPC) of the row is set.
// The second one only matters to the transposing loader, whose 16 lanes of one LDS access write rows
// r and r + EPC: without it both rows would sit in the same half of the banks.
template <typename T>
__device__ __forceinline__ int lds_row(int row) {
  constexpr int BIT = sizeof(T) == 2 ? 3 : 2;
  return row ^ ((row >> BIT) & 1);
}
template <typename T>
__device__ __forceinline__ int lds_off(int row, int q) {
  return lds_row<T>(row) * 128 + ((q ^ ((row >> 1) & 7)) << 4);
}

// Sixteen zero bytes in device memory: out-of-range pieces are redirected here, so that the loaded
// value needs no masking (a select on loaded data would force the wave to wait for the load at once).
__device__ const uint4 kZeroChunk = {0u, 0u, 0u, 0u};

// Loads and stores go through pointers that carry the global address space explicitly: a generic
// ("flat") access would also count against the LDS counter and make every wait for an LDS read wait
// for HBM as well.
template <typename V>
__device__ __forceinline__ V global_load(uintptr_t addr) {
  return *reinterpret_cast<const __attribute__((address_space(1))) V *>(addr);
}
template <typename V>
__device__ __forceinline__ void global_store(uintptr_t addr, V v) {
  *reinterpret_cast<__attribute__((address_space(1))) V *>(addr) = v;
}

// Load one 16-byte chunk starting at address p in pieces of PB bytes without any branch: a piece
// whose first element index is >= n_valid is read from the zero chunk instead.  Pieces never straddle
// the valid range because the host only picks a piece size that divides the operand's extent along
// its unit-stride dimension.
template <typename T, int PB>
__device__ __forceinline__ uint4 load_chunk(uintptr_t p, int n_valid) {
  constexpr int PE = PB / (int)sizeof(T);   // elements per piece
  constexpr int NP = 16 / PB;               // pieces per chunk
  const uintptr_t zero = reinterpret_cast<uintptr_t>(&kZeroChunk);
  uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int j = 0; j < NP; ++j) {
    const uintptr_t q = (j * PE < n_valid) ? p + j * PB : zero;
    if constexpr (PB == 16) {
      const u32x4 v = global_load<u32x4>(q);
      w[0] = v[0]; w[1] = v[1]; w[2] = v[2]; w[3] = v[3];
    } else if constexpr (PB == 8) {
      const u32x2 v = global_load<u32x2>(q);
      w[2 * j] = v[0]; w[2 * j + 1] = v[1];
    } else if constexpr (PB == 4) {
      w[j] = global_load<uint32_t>(q);
    } else {
      const uint32_t v = global_load<uint16_t>(q);
      w[j >> 1] |= v << ((j & 1) * 16);
    }
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

// One operand tile: ROWS rows (m or n) x 128 bytes of k, staged in registers between global memory
// and LDS.  Everything that does not change from tile step to tile step (slot addresses, row
// validity) is computed once in init().
template <typename T, int ROWS, bool KC, int PB>
struct TileLoader {
  static constexpr int EPC = Traits<T>::EPC;
  static constexpr int NS = ROWS / 32;                      // ROWS * 8 chunks / 256 threads
  static constexpr int NBLK = 8 * ROWS / EPC;               // EPC x EPC transpose blocks per tile
  static constexpr int NB = (NBLK + 255) / 256;             // ... per thread
  static constexpr int NSLOT = KC ? NS : NB;
  uint4 reg[KC ? NS : NB * EPC];
  uintptr_t ptr[NSLOT];   // address of the slot's first element for k0 = 0
  int lim[NSLOT];         // KC: K - (k offset of the slot) for valid rows, else 0;  MC: rows_total - m or 0
  int64_t kstride;        // bytes between consecutive k (MC only)
  int K;
  uintptr_t pf_ptr;       // cache-line prefetch: this thread's line of the tile at k0 = 0
  int pf_lim;             // KC: K if the thread's row exists, else 0;  MC: K - (its k row) or 0

  __device__ __forceinline__ void init(const T *base, int64_t ld, int rows_total, int row0, int K_) {
    K = K_;
    kstride = ld * (int64_t)sizeof(T);
    if constexpr (KC) {   // one 128-byte line per tile row: thread t takes row t
      const int row = row0 + (int)threadIdx.x;
      pf_ptr = reinterpret_cast<uintptr_t>(base + (int64_t)row * ld);
      pf_lim = (threadIdx.x < ROWS && row < rows_total) ? K_ : 0;
    } else {              // ROWS * sizeof(T) / 128 lines per k row
      constexpr int LPR = ROWS * (int)sizeof(T) / 128, EPL = 128 / (int)sizeof(T);
      const int kr = threadIdx.x / LPR, m = row0 + (threadIdx.x % LPR) * EPL;
      pf_ptr = reinterpret_cast<uintptr_t>(base + (int64_t)kr * ld + m);
      pf_lim = (kr < 128 / (int)sizeof(T) && m < rows_total) ? K_ - kr : 0;
    }
    if constexpr (KC) {
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        const int s = threadIdx.x + i * 256;
        const int row = row0 + (s >> 3), kc = (s & 7) * EPC;
        ptr[i] = reinterpret_cast<uintptr_t>(base + (int64_t)row * ld + kc);
        lim[i] = row < rows_total ? K - kc : 0;
      }
    } else {
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const int blk = threadIdx.x + b * 256;
        const int kg = blk & 7, mc = blk >> 3;
        const int m = row0 + mc * EPC;
        ptr[b] = reinterpret_cast<uintptr_t>(base + (int64_t)(kg * EPC) * ld + m);
        lim[b] = blk < NBLK ? rows_total - m : 0;
      }
    }
  }

  // issue the global loads of the tile whose first k is k0
  __device__ __forceinline__ void issue(int k0) {
    if constexpr (KC) {
#pragma unroll
      for (int i = 0; i < NS; ++i)
        reg[i] = load_chunk<T, PB>(ptr[i] + (int64_t)k0 * (int64_t)sizeof(T), lim[i] - k0);
    } else {
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const int kg = (threadIdx.x + b * 256) & 7;
#pragma unroll
        for (int j = 0; j < EPC; ++j) {
          const int k = k0 + kg * EPC + j;
          reg[b * EPC + j] = load_chunk<T, PB>(ptr[b] + (int64_t)(k0 + j) * kstride, k < K ? lim[b] : 0);
        }
      }
    }
  }

  // Touch this thread's cache line of the tile whose first k is k0, so that the line is on its way
  // into L2 long before the tile's real loads are issued.  The value is meaningless.
  __device__ __forceinline__ uint32_t prefetch(int k0) const {
    const uintptr_t zero = reinterpret_cast<uintptr_t>(&kZeroChunk);
    const uintptr_t a = KC ? pf_ptr + (int64_t)k0 * (int64_t)sizeof(T) : pf_ptr + (int64_t)k0 * kstride;
    return global_load<uint32_t>(k0 < pf_lim ? a : zero);
  }

  __device__ __forceinline__ void store(char *lds) const {
    if constexpr (KC) {
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        const int s = threadIdx.x + i * 256;
        *reinterpret_cast<uint4 *>(lds + lds_off<T>(s >> 3, s & 7)) = reg[i];
      }
    } else {
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const int blk = threadIdx.x + b * 256;
        if constexpr (NBLK % 256 != 0) {   // only small tiles have idle threads here; a branch in the
          if (blk >= NBLK) continue;       // big tile's loop would split its scheduling region
        }
        const int kg = blk & 7, mc = blk >> 3;
        const uint4 *r = &reg[b * EPC];
#pragma unroll
        for (int e = 0; e < EPC; ++e) {
          uint4 o;
          if constexpr (sizeof(T) == 4) {
            o = make_uint4((&r[0].x)[e], (&r[1].x)[e], (&r[2].x)[e], (&r[3].x)[e]);
          } else {
            uint32_t w[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              // one byte permute per output word: low halves (even e) or high halves (odd e) of lo, hi
              const uint32_t lo = (&r[2 * q].x)[e >> 1], hi = (&r[2 * q + 1].x)[e >> 1];
              w[q] = __builtin_amdgcn_perm(hi, lo, (e & 1) ? 0x07060302u : 0x05040100u);
            }
            o = make_uint4(w[0], w[1], w[2], w[3]);
          }
          *reinterpret_cast<uint4 *>(lds + lds_off<T>(mc * EPC + e, kg)) = o;
        }
      }
    }
  }
};

// MFMA operand fragments of one k-step: one 16-byte chunk per 32 rows of A and of B.
template <int TM, int TN>
struct Frags {
  uint4 a[TM], b[TN];
  // sa / sb: this lane's row inside the wave's A / B rows of the stage; off: swizzled chunk offset
  __device__ __forceinline__ void read(const char *sa, const char *sb, int off) {
#pragma unroll
    for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const uint4 *>(sa + i * (32 * 128) + off);
#pragma unroll
    for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const uint4 *>(sb + j * (32 * 128) + off);
  }
};

template <typename T, int TM, int TN>
__device__ __forceinline__ void mma(floatx16 (&acc)[TM][TN], const Frags<TM, TN> &f) {
  if constexpr (sizeof(T) == 2) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f.a[i]),
                                                            __builtin_bit_cast(bf16x8, f.b[j]), acc[i][j], 0, 0, 0);
  } else {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float((&f.a[i].x)[kk]),
                                                           __uint_as_float((&f.b[j].x)[kk]), acc[i][j], 0, 0, 0);
  }
}

// Scheduling hints (instruction-class masks of __builtin_amdgcn_sched_group_barrier).
constexpr int SG_MFMA = 0x008, SG_VMEM_READ = 0x020, SG_DS_READ = 0x100, SG_DS_WRITE = 0x200;

// `groups` times: `nr` LDS reads, then `nm` MFMAs.
template <int GROUPS, int NR, int NM>
__device__ __forceinline__ void sched_reads_mfma() {
#pragma unroll
  for (int g = 0; g < GROUPS; ++g) {
    __builtin_amdgcn_sched_group_barrier(SG_DS_READ, NR, 0);
    __builtin_amdgcn_sched_group_barrier(SG_MFMA, NM, 0);
  }
}

// ---- epilogue helpers ------------------------------------------------------------------------------
// Two paths.  The fast one handles whole 4-column groups with aligned vector accesses only (the host
// sets epi_vec when every pointer and leading dimension allows it) and keeps its code small because
// it is replicated for every row segment a lane owns; everything else (ragged right edge, unaligned
// views) goes through a rolled element-by-element loop.
struct Vec4 { float v[4]; };

__device__ __forceinline__ Vec4 load4v(const void *p, int64_t idx, int is_bf16) {
  Vec4 r;
  if (is_bf16) {
    const u32x2 w = global_load<u32x2>(reinterpret_cast<uintptr_t>(static_cast<const bf16_raw *>(p) + idx));
    r.v[0] = __uint_as_float(w[0] << 16); r.v[1] = __uint_as_float(w[0] & 0xffff0000u);
    r.v[2] = __uint_as_float(w[1] << 16); r.v[3] = __uint_as_float(w[1] & 0xffff0000u);
  } else {
    const f32x4 w = global_load<f32x4>(reinterpret_cast<uintptr_t>(static_cast<const float *>(p) + idx));
    r.v[0] = w[0]; r.v[1] = w[1]; r.v[2] = w[2]; r.v[3] = w[3];
  }
  return r;
}

__device__ __forceinline__ void store4v(void *p, int64_t idx, int is_bf16, const Vec4 &x) {
  if (is_bf16) {
    u32x2 w;
    w[0] = (uint32_t)f32_to_bf16(x.v[0]) | ((uint32_t)f32_to_bf16(x.v[1]) << 16);
    w[1] = (uint32_t)f32_to_bf16(x.v[2]) | ((uint32_t)f32_to_bf16(x.v[3]) << 16);
    global_store<u32x2>(reinterpret_cast<uintptr_t>(static_cast<bf16_raw *>(p) + idx), w);
  } else {
    f32x4 w = {x.v[0], x.v[1], x.v[2], x.v[3]};
    global_store<f32x4>(reinterpret_cast<uintptr_t>(static_cast<float *>(p) + idx), w);
  }
}

__device__ __forceinline__ float load1(const void *p, int64_t idx, int is_bf16) {
  return is_bf16 ? bf16_to_f32(static_cast<const bf16_raw *>(p)[idx]) : static_cast<const float *>(p)[idx];
}
__device__ __forceinline__ void store1(void *p, int64_t idx, int is_bf16, float v) {
  if (is_bf16) static_cast<bf16_raw *>(p)[idx] = f32_to_bf16(v);
  else static_cast<float *>(p)[idx] = v;
}

// alpha/beta, bias, activation or activation gradient for one value; c0 = old C, aux = retained
// activation (both only read when the epilogue uses them).  Returns the pre-activation through *pre.
__device__ __forceinline__ float epi_math(const GemmArgs &g, float acc, float c0, float bias, float aux, float *pre) {
  float x = g.alpha * acc;
  if (g.beta != 0.0f) x += g.beta * c0;
  x += bias;
  *pre = x;
  if (g.epi == CHN_EPI_BIAS_RELU) x = fmaxf(x, 0.0f);
  else if (g.epi == CHN_EPI_BIAS_GELU) x = gelu_epi_f(x);
  else if (g.epi == CHN_EPI_RELU_BWD) x = aux > 0.0f ? x : 0.0f;
  else if (g.epi == CHN_EPI_GELU_BWD) x *= gelu_grad_epi_f(aux);
  return x;
}

// The fast path's dependent global reads (C when beta != 0, aux for the activation gradients) for
// the four columns col.. of row `row`.  They are issued for several row segments at once before any
// of them is used: a wave that is alone on its SIMD would otherwise sit out one memory latency per
// segment.
struct EpiIn { Vec4 c0, aux; };

__device__ __forceinline__ EpiIn epi_fetch(const GemmArgs &g, int row, int col) {
  EpiIn in;
#pragma unroll
  for (int e = 0; e < 4; ++e) in.c0.v[e] = in.aux.v[e] = 0.0f;
  if (g.beta != 0.0f) in.c0 = load4v(g.C, (int64_t)row * g.ldc + col, g.c_bf16);
  if (g.epi == CHN_EPI_RELU_BWD || g.epi == CHN_EPI_GELU_BWD) in.aux = load4v(g.aux, (int64_t)row * g.ldaux + col, g.c_bf16);
  return in;
}

__device__ __forceinline__ void finish4(const GemmArgs &g, int row, int col, const f32x4 a, const EpiIn &in) {
  Vec4 b, x, pre;
#pragma unroll
  for (int e = 0; e < 4; ++e) b.v[e] = 0.0f;
  if (g.epi >= CHN_EPI_BIAS && g.epi <= CHN_EPI_BIAS_GELU) b = load4v(g.bias, col, 0);
#pragma unroll
  for (int e = 0; e < 4; ++e) x.v[e] = epi_math(g, a[e], in.c0.v[e], b.v[e], in.aux.v[e], &pre.v[e]);
  if (g.epi == CHN_EPI_BIAS_GELU && g.pre) store4v(g.pre, (int64_t)row * g.ldpre + col, g.c_bf16, pre);
  store4v(g.C, (int64_t)row * g.ldc + col, g.c_bf16, x);
}

// One element, any alignment (slow path).
__device__ __forceinline__ void finish1(const GemmArgs &g, int row, int col, float acc) {
  const int64_t ci = (int64_t)row * g.ldc + col;
  const float c0 = g.beta != 0.0f ? load1(g.C, ci, g.c_bf16) : 0.0f;
  const float bias = (g.epi >= CHN_EPI_BIAS && g.epi <= CHN_EPI_BIAS_GELU) ? g.bias[col] : 0.0f;
  const float aux = (g.epi == CHN_EPI_RELU_BWD || g.epi == CHN_EPI_GELU_BWD) ? load1(g.aux, (int64_t)row * g.ldaux + col, g.c_bf16) : 0.0f;
  float pre;
  const float x = epi_math(g, acc, c0, bias, aux, &pre);
  if (g.epi == CHN_EPI_BIAS_GELU && g.pre) store1(g.pre, (int64_t)row * g.ldpre + col, g.c_bf16, pre);
  store1(g.C, ci, g.c_bf16, x);
}

// Rows [row0, row0+32) x columns [col0, col0 + 32*TN) of C for one wave: `stage` holds the fp32
// accumulators row-major with pitch PITCH floats.  With K splits the raw sums go to this split's
// slab of the workspace instead.
template <int TN>
__device__ __forceinline__ void epilogue_rows(const GemmArgs &g, const float *stage, int row0, int col0, int lane, float *slab) {
  constexpr int W = 32 * TN, PITCH = W + 8, CPR = W / 4;      // 16-byte chunks per row
  constexpr int NIT = 32 * CPR / 64;                          // row segments per lane
  constexpr int U = NIT < 4 ? NIT : 4;                        // segments whose reads are in flight together
  if (slab) {                                                 // split-K: raw sums, always aligned (ldp % 4 == 0)
    for (int c = lane; c < 32 * CPR; c += 64) {
      const int rl = c / CPR, cl = (c % CPR) * 4;
      if (row0 + rl < g.M && col0 + cl < g.N)
        global_store<f32x4>(reinterpret_cast<uintptr_t>(slab + (int64_t)(row0 + rl) * g.ldp + col0 + cl),
                            *reinterpret_cast<const f32x4 *>(stage + rl * PITCH + cl));
    }
  } else if (g.epi_vec && col0 + W <= g.N) {                  // fast path: lane l handles 4 consecutive columns
#pragma unroll 1
    for (int base = 0; base < NIT; base += U) {
      EpiIn in[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int c = lane + (base + u) * 64;
        if (row0 + c / CPR < g.M) in[u] = epi_fetch(g, row0 + c / CPR, col0 + (c % CPR) * 4);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int c = lane + (base + u) * 64;
        const int rl = c / CPR, cl = (c % CPR) * 4;
        if (row0 + rl < g.M) finish4(g, row0 + rl, col0 + cl, *reinterpret_cast<const f32x4 *>(stage + rl * PITCH + cl), in[u]);
      }
    }
  } else {                                                    // slow path: one element at a time
#pragma unroll 1
    for (int c = lane; c < 32 * W; c += 64) {
      const int rl = c / W, cl = c % W;
      if (row0 + rl < g.M && col0 + cl < g.N) finish1(g, row0 + rl, col0 + cl, stage[rl * PITCH + cl]);
    }
  }
}

// Second kernel of a split product: adds the slabs in split order and runs the epilogue.
static __global__ __launch_bounds__(256) void gemm_splitk_finish_kernel(GemmArgs g) {
  const int groups = (int)(g.ldp / 4);
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= (int64_t)g.M * groups) return;
  const int row = (int)(e / groups), col = (int)(e % groups) * 4;
  if (col >= g.N) return;
  const int64_t slab = (int64_t)g.M * g.ldp;
  const float *p = g.partial + (int64_t)row * g.ldp + col;
  f32x4 a = global_load<f32x4>(reinterpret_cast<uintptr_t>(p));
  for (int s = 1; s < g.splits; ++s) a += global_load<f32x4>(reinterpret_cast<uintptr_t>(p + s * slab));
  if (g.epi_vec && col + 4 <= g.N) {
    finish4(g, row, col, a, epi_fetch(g, row, col));
  } else {
    for (int e = 0; e < 4 && col + e < g.N; ++e) finish1(g, row, col + e, a[e]);
  }
}

template <typename T, int TM, int TN, bool A_KC, bool B_KC, int PB>
__global__ __launch_bounds__(256) void gemm_kernel(GemmArgs g) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  constexpr int BK = 128 / sizeof(T);               // elements of k per tile step
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
  extern __shared__ __align__(16) char lds[];

  // ---- which C tile: XCD-aware renumbering, then grouped (8 tile rows at a time) ordering
  const int nb = g.tiles_m * g.tiles_n;
  int pid = blockIdx.x % nb;
  const int split = blockIdx.x / nb;
  const int nb8 = nb & ~7;
  if (pid < nb8) pid = (pid & 7) * (nb8 >> 3) + (pid >> 3);
  constexpr int GROUP = 8;
  const int width = GROUP * g.tiles_n;
  const int first_m = (pid / width) * GROUP;
  const int gsize = min(g.tiles_m - first_m, GROUP);
  const int tm = first_m + (pid % width) % gsize;
  const int tn = (pid % width) / gsize;
  const int m0 = tm * BM, n0 = tn * BN;

  TileLoader<T, BM, A_KC, PB> la;
  TileLoader<T, BN, B_KC, PB> lb;
  la.init(static_cast<const T *>(g.A), g.lda, g.M, m0, g.K);
  lb.init(static_cast<const T *>(g.B), g.ldb, g.N, n0, g.K);

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const int r = lane & 31, h = lane >> 5;

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  // byte offsets of this lane's fragment rows inside a stage, and of its chunk per k-step
  const int rp = lds_row<T>(r);
  const int a_row = (wm * TM * 32 + rp) * 128, b_row = A_BYTES + (wn * TN * 32 + rp) * 128;
  const int sw = (r >> 1) & 7;
  int koff[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) koff[ks] = ((ks * 2 + h) ^ sw) << 4;

  // this block's range of tile steps along K (all of them unless the product is split)
  const int nk_all = (g.K + BK - 1) / BK;
  const int per_split = (nk_all + g.splits - 1) / g.splits;
  const int kt0 = split * per_split;
  const int nk = min(nk_all, kt0 + per_split);
  la.issue(kt0 * BK);
  lb.issue(kt0 * BK);
  la.store(lds);
  lb.store(lds + A_BYTES);
  __syncthreads();
  Frags<TM, TN> f0, f1;
  f0.read(lds + a_row, lds + b_row, koff[0]);

  uint32_t pf_a = 0, pf_b = 0;
  constexpr int kPrefetchAhead = 3;
  constexpr int NM = (sizeof(T) == 2 ? 1 : 4) * TM * TN;   // MFMAs per k-step
  constexpr int NR = TM + TN;                              // fragment reads per k-step
  constexpr bool kSched = TM == 4 && TN == 4;              // explicit interleaving for the big tile

  for (int kt = kt0; kt < nk; ++kt) {
    const char *cur = lds + ((kt - kt0) & 1) * STAGE;
    char *nxt = lds + ((kt - kt0 + 1) & 1) * STAGE;
    // k-step 0, overlapped with the issue of the global loads of the next tile (they are written to
    // LDS in k-step 2; keeping issue and use inside one loop iteration keeps the staging registers
    // from being carried -- and copied, which means waited for -- across the loop's back edge)
    f1.read(cur + a_row, cur + b_row, koff[1]);
    la.issue((kt + 1) * BK);
    lb.issue((kt + 1) * BK);
    mma<T, TM, TN>(acc, f0);
    if constexpr (kSched) {
#pragma unroll
      for (int s = 0; s < NR; ++s) {
        __builtin_amdgcn_sched_group_barrier(SG_DS_READ, 1, 0);
        __builtin_amdgcn_sched_group_barrier(SG_VMEM_READ, 2 * (16 / PB), 0);
        __builtin_amdgcn_sched_group_barrier(SG_MFMA, NM / NR, 0);
      }
    }
    // k-step 1 (the big tile also touches the cache lines of the tile three steps ahead: with one wave
    // per SIMD the two k-steps between issue and use of a tile's loads cover an L2 hit, not HBM)
    f0.read(cur + a_row, cur + b_row, koff[2]);
    if constexpr (kSched) {
      asm volatile("" ::"v"(pf_a), "v"(pf_b));   // the previous touches must not be optimised away
      pf_a = la.prefetch((kt + kPrefetchAhead) * BK);
      pf_b = lb.prefetch((kt + kPrefetchAhead) * BK);
    }
    mma<T, TM, TN>(acc, f1);
    if constexpr (kSched) sched_reads_mfma<NR, 1, NM / NR>();
    // k-step 2: also move the next tile from registers to the other stage.  The compiler must keep
    // every LDS read ahead of every LDS write (it cannot tell the two stages apart), so the reads
    // pair with the first half of the MFMAs and the writes with the second half.
    f1.read(cur + a_row, cur + b_row, koff[3]);
    if constexpr (A_KC) la.store(nxt);
    if constexpr (B_KC) lb.store(nxt + A_BYTES);
    mma<T, TM, TN>(acc, f0);
    if constexpr (kSched) {
      constexpr int NW = (A_KC ? TM * 2 : 0) + (B_KC ? TN * 2 : 0);   // 16-byte LDS writes interleaved
      sched_reads_mfma<NR, 1, NM / NR / 2>();
#pragma unroll
      for (int s = 0; s < NR; ++s) {
        __builtin_amdgcn_sched_group_barrier(SG_DS_WRITE, NW / NR, 0);
        __builtin_amdgcn_sched_group_barrier(SG_MFMA, NM / NR / 2, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    // A transposed operand's first LDS write needs all of its loads (an 8x8 block is transposed in
    // registers), so its wait would stall the MFMAs queued behind it: those writes go last.
    if constexpr (!A_KC) la.store(nxt);
    if constexpr (!B_KC) lb.store(nxt + A_BYTES);
    __syncthreads();
    // k-step 3, overlapped with the first fragment reads of the next stage
    f0.read(nxt + a_row, nxt + b_row, koff[0]);
    mma<T, TM, TN>(acc, f1);
    if constexpr (kSched) sched_reads_mfma<NR, 1, NM / NR>();
  }

  // ---- epilogue: per wave and per 32-row block, accumulators -> LDS (row-major) -> vector epilogue.
  // Lane holds, per 32x32 block, column r and rows 8*(v/4) + 4*h + v%4.
  __syncthreads();   // every wave is done with the operand stages
  constexpr int PITCH = 32 * TN + 8;
  float *stage = reinterpret_cast<float *>(lds) + wave * (32 * PITCH);
  float *slab = g.splits > 1 ? g.partial + (int64_t)split * g.M * g.ldp : nullptr;
  // (written out per 32-row block: the compiler refuses to unroll a loop this large, and a rolled
  // loop would index the accumulator registers dynamically, i.e. move them to scratch memory)
  auto block = [&](auto ic) {
    constexpr int i = decltype(ic)::value;
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) stage[(8 * (v >> 2) + 4 * h + (v & 3)) * PITCH + j * 32 + r] = acc[i][j][v];
    __builtin_amdgcn_wave_barrier();
    epilogue_rows<TN>(g, stage, m0 + (wm * TM + i) * 32, n0 + wn * TN * 32, lane, slab);
    __builtin_amdgcn_wave_barrier();
  };
  block(std::integral_constant<int, 0>{});
  if constexpr (TM > 1) block(std::integral_constant<int, 1>{});
  if constexpr (TM > 2) {
    block(std::integral_constant<int, 2>{});
    block(std::integral_constant<int, 3>{});
  }
}

template <typename T, int TM, int TN, bool A_KC, bool B_KC, int PB>
chn_status launch_piece(const GemmArgs &g, hipStream_t st) {
  constexpr int LDS = 2 * (64 * TM + 64 * TN) * 128;
  static_assert(4 * 32 * (32 * TN + 8) * 4 <= LDS, "epilogue staging must fit in the operand stages");
  auto kern = gemm_kernel<T, TM, TN, A_KC, B_KC, PB>;
  static bool configured = false;  // per instantiation
  if (!configured) {
    if (LDS > 64 * 1024) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
      if (e != hipSuccess) return fail(CHN_ERR_LAUNCH, "gemm: cannot reserve %d bytes of LDS: %s", LDS, hipGetErrorString(e));
    }
    configured = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)(g.tiles_m * g.tiles_n * g.splits)), dim3(256), LDS, st, g);
  CHN_TRY(check_launch("gemm"));
  if (g.splits > 1) {
    const int64_t n = (int64_t)g.M * (g.ldp / 4);
    hipLaunchKernelGGL(gemm_splitk_finish_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, g);
    return check_launch("gemm split-K finish");
  }
  return CHN_OK;
}

template <typename T, int TM, int TN, bool A_KC, bool B_KC>
chn_status launch_tile(const GemmArgs &g, hipStream_t st) {
  if (g.piece == 16) return launch_piece<T, TM, TN, A_KC, B_KC, 16>(g, st);
  if (g.piece == 8) return launch_piece<T, TM, TN, A_KC, B_KC, 8>(g, st);
  if constexpr (TM == 1) return launch_piece<T, 1, 1, A_KC, B_KC, (int)sizeof(T)>(g, st);
  else return fail(CHN_ERR_LAUNCH, "gemm: internal: element-wise loads only exist for the 64x64 tile");
}

template <typename T, bool A_KC, bool B_KC>
chn_status launch_layout(GemmArgs &g, hipStream_t st) {
  if ((int64_t)g.tiles_m * g.tiles_n * g.splits > 0x7fffffff) return fail(CHN_ERR_SHAPE, "gemm: too many tiles");
  if (g.tile == 2) return launch_tile<T, 4, 4, A_KC, B_KC>(g, st);
  if (g.tile == 1) return launch_tile<T, 2, 2, A_KC, B_KC>(g, st);
  return launch_tile<T, 1, 1, A_KC, B_KC>(g, st);
}

}  // namespace gemm
}  // namespace chn
