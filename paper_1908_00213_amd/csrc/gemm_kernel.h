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
// whose first element index is >= n_valid is read from the zero chunk instead.  Along K a piece never
// straddles the valid range, because there the host only picks a piece size that divides the operand's
// extent; along M or N the last piece of a row may bring elements from beyond the row's end, which
// only ever reach rows or columns of C that are not stored.
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
  // A 64-row tile with unit stride along M/N has fewer transpose blocks (EPC k x EPC m) than the
  // workgroup has threads: 64 of bf16, 128 of fp32.  Every load instruction of a wave costs the memory
  // pipeline the same whether its lanes fetch data or are parked on the zero chunk, so CP = 4 (2)
  // threads share a block instead: each loads two of its k-rows and writes, for every m, the 4 (8)
  // bytes -- two k -- it can form.  A wave takes all eight k-groups of 2 (4) m-chunks, which spreads
  // its narrow LDS writes over all banks, two lanes each.
  static constexpr bool COOP = !KC && ROWS == 64;
  static constexpr int CP = COOP ? 256 / NBLK : 1;
  static constexpr int NSLOT = KC ? NS : NB;
  uint4 reg[2][KC ? NS : COOP ? 2 : NB * EPC];   // two sets of staging registers (the second only where a kernel looks two tiles ahead)
  uintptr_t ptr[NSLOT];   // address of the slot's first element for k0 = 0
  int lim[NSLOT];         // KC: K - (k offset of the slot) for valid rows, else 0;  MC: rows_total - m or 0
  int64_t kstride;        // bytes between consecutive k (MC only)
  int K;
  uintptr_t pf_ptr;       // cache-line prefetch: this thread's line of the tile at k0 = 0
  int pf_lim;             // KC: K if the thread's row exists, else 0;  MC: K - (its k row) or 0
  int tid;                // MC: the thread's number in the dealing of transpose blocks

  // shift: a small tile has fewer transpose blocks than the workgroup has threads (64 for 64 rows of
  // bf16: one wave's worth); rotating the dealing by `shift` threads puts the second operand's blocks
  // on waves -- and so on SIMDs -- that the first operand's leave idle.
  __device__ __forceinline__ void init(const T *base, int64_t ld, int rows_total, int row0, int K_, int shift = 0) {
    K = K_;
    tid = ((int)threadIdx.x + shift) & 255;
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
    } else if constexpr (COOP) {
      const int m = row0 + coop_mc() * EPC;
      ptr[0] = reinterpret_cast<uintptr_t>(base + (int64_t)(coop_kg() * EPC + 2 * coop_part()) * ld + m);
      lim[0] = rows_total - m;
    } else {
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const int blk = tid + b * 256;
        const int kg = blk & 7, mc = blk >> 3;
        const int m = row0 + mc * EPC;
        ptr[b] = reinterpret_cast<uintptr_t>(base + (int64_t)(kg * EPC) * ld + m);
        lim[b] = blk < NBLK ? rows_total - m : 0;
      }
    }
  }
  // COOP: which quarter (two k-rows) of which block (k-group, m-chunk) the thread handles
  __device__ __forceinline__ int coop_part() const { return threadIdx.x % CP; }
  __device__ __forceinline__ int coop_kg() const { return (threadIdx.x / CP) & 7; }
  __device__ __forceinline__ int coop_mc() const { return (8 / CP) * (threadIdx.x >> 6) + (threadIdx.x & 63) / (8 * CP); }

  // issue the global loads of the tile whose first k is k0 (into register set SET)
  template <int SET = 0>
  __device__ __forceinline__ void issue(int k0) {
    if constexpr (KC) {
#pragma unroll
      for (int i = 0; i < NS; ++i)
        reg[SET][i] = load_chunk<T, PB>(ptr[i] + (int64_t)k0 * (int64_t)sizeof(T), lim[i] - k0);
    } else if constexpr (COOP) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int k = k0 + coop_kg() * EPC + 2 * coop_part() + j;
        reg[SET][j] = load_chunk<T, PB>(ptr[0] + (int64_t)(k0 + j) * kstride, k < K ? lim[0] : 0);
      }
    } else {
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const int kg = (tid + b * 256) & 7;
#pragma unroll
        for (int j = 0; j < EPC; ++j) {
          const int k = k0 + kg * EPC + j;
          reg[SET][b * EPC + j] = load_chunk<T, PB>(ptr[b] + (int64_t)(k0 + j) * kstride, k < K ? lim[b] : 0);
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

  template <int SET = 0>
  __device__ __forceinline__ void store(char *lds) const {
    if constexpr (KC) {
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        const int s = threadIdx.x + i * 256;
        *reinterpret_cast<uint4 *>(lds + lds_off<T>(s >> 3, s & 7)) = reg[SET][i];
      }
    } else if constexpr (COOP) {
      const int kg = coop_kg(), row0l = coop_mc() * EPC, part = coop_part();
#pragma unroll
      for (int e = 0; e < EPC; ++e) {
        // k = 2 part and 2 part + 1 of row m = e of the block
        char *q = lds + lds_off<T>(row0l + e, kg);
        if constexpr (sizeof(T) == 2) {
          const uint32_t lo = (&reg[SET][0].x)[e >> 1], hi = (&reg[SET][1].x)[e >> 1];
          *reinterpret_cast<uint32_t *>(q + part * 4) = __builtin_amdgcn_perm(hi, lo, (e & 1) ? 0x07060302u : 0x05040100u);
        } else {
          *reinterpret_cast<uint2 *>(q + part * 8) = make_uint2((&reg[SET][0].x)[e], (&reg[SET][1].x)[e]);
        }
      }
    } else {
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const int blk = tid + b * 256;
        if constexpr (NBLK % 256 != 0) {   // only small tiles have idle threads here; a branch in the
          if (blk >= NBLK) continue;       // big tile's loop would split its scheduling region
        }
        const int kg = blk & 7, mc = blk >> 3;
        const uint4 *r = &reg[SET][b * EPC];
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
constexpr int SG_MFMA = 0x008, SG_VMEM = 0x010, SG_VMEM_READ = 0x020, SG_DS_READ = 0x100, SG_DS_WRITE = 0x200;
// s_waitcnt immediate (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8) that waits
// for the vector-memory counter only.
constexpr int kWaitVmcnt0 = 0x0F70;

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
// it is replicated for every row segment a lane owns; a pass that crosses the last row or column of
// aligned operands runs a rolled loop over the 4-column groups that lie in range, and unaligned views
// go through a rolled element-by-element loop.
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
  else if (g.epi == CHN_EPI_BIAS_GELU) x = g.c_bf16 ? gelu_epi_bf16_f(x) : gelu_epi_f(x);
  else if (g.epi == CHN_EPI_RELU_BWD) x = aux > 0.0f ? x : 0.0f;
  else if (g.epi == CHN_EPI_GELU_BWD) x *= g.c_bf16 ? gelu_grad_epi_bf16_f(aux) : gelu_grad_epi_f(aux);
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
  if (g.epi == CHN_EPI_BF16_COPY) store4v(g.pre, (int64_t)row * g.ldpre + col, 1, x);
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
  if (g.epi == CHN_EPI_BF16_COPY) store1(g.pre, (int64_t)row * g.ldpre + col, 1, x);
  store1(g.C, ci, g.c_bf16, x);
}

// Four elements of C's dtype as they come from memory; converted only where they are used, so that
// issuing the load does not tie the wave to its arrival.
template <bool CB> struct Raw4 { typedef f32x4 type; };
template <> struct Raw4<true> { typedef u32x2 type; };
template <bool CB>
__device__ __forceinline__ typename Raw4<CB>::type load4raw(const void *p, int64_t idx) {
  if constexpr (CB) return global_load<u32x2>(reinterpret_cast<uintptr_t>(static_cast<const bf16_raw *>(p) + idx));
  else return global_load<f32x4>(reinterpret_cast<uintptr_t>(static_cast<const float *>(p) + idx));
}
__device__ __forceinline__ Vec4 cvt4(const u32x2 w) {
  Vec4 r;
  r.v[0] = __uint_as_float(w[0] << 16); r.v[1] = __uint_as_float(w[0] & 0xffff0000u);
  r.v[2] = __uint_as_float(w[1] << 16); r.v[3] = __uint_as_float(w[1] & 0xffff0000u);
  return r;
}
__device__ __forceinline__ Vec4 cvt4(const f32x4 w) {
  Vec4 r;
  r.v[0] = w[0]; r.v[1] = w[1]; r.v[2] = w[2]; r.v[3] = w[3];
  return r;
}
template <bool CB> struct EpiRaw { typename Raw4<CB>::type c0, aux; };

// Same as finish4 with the epilogue kind, C's dtype (CB: bf16) and whether old C is added (BETA) fixed
// at compile time (the tile kernels pick them once per pass, outside their loops, which are then free
// of branches).
// (*stored, if not null, receives the four values as C holds them, i.e. after rounding to its dtype)
template <int EPI, bool CB, bool BETA>
__device__ __forceinline__ void finish4_t(const GemmArgs &g, int row, int col, const f32x4 a, const EpiRaw<CB> &raw, const Vec4 &b,
                                          Vec4 *stored = nullptr) {
  Vec4 x, pre;
  EpiIn in;
  if constexpr (BETA) in.c0 = cvt4(raw.c0);
  if constexpr (EPI == CHN_EPI_RELU_BWD || EPI == CHN_EPI_GELU_BWD) in.aux = cvt4(raw.aux);
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    float t = g.alpha * a[e];
    if constexpr (BETA) t += g.beta * in.c0.v[e];
    t += b.v[e];
    pre.v[e] = t;
    if constexpr (EPI == CHN_EPI_BIAS_RELU) t = fmaxf(t, 0.0f);
    else if constexpr (EPI == CHN_EPI_BIAS_GELU) t = CB ? gelu_epi_bf16_f(t) : gelu_epi_f(t);
    else if constexpr (EPI == CHN_EPI_RELU_BWD) t = in.aux.v[e] > 0.0f ? t : 0.0f;
    else if constexpr (EPI == CHN_EPI_GELU_BWD) t *= CB ? gelu_grad_epi_bf16_f(in.aux.v[e]) : gelu_grad_epi_f(in.aux.v[e]);
    x.v[e] = t;
  }
  if constexpr (EPI == CHN_EPI_BIAS_GELU) {
    if (g.pre) store4v(g.pre, (int64_t)row * g.ldpre + col, CB, pre);
  }
  if constexpr (EPI == CHN_EPI_BF16_COPY) store4v(g.pre, (int64_t)row * g.ldpre + col, true, x);
  store4v(g.C, (int64_t)row * g.ldc + col, CB, x);
  if (stored) {
#pragma unroll
    for (int e = 0; e < 4; ++e) stored->v[e] = CB ? bf16_to_f32(f32_to_bf16(x.v[e])) : x.v[e];
  }
}

// Where the accumulators of one wave wait in LDS between the MFMA register layout and the row-major
// epilogue: RP rows of W = 32*TN floats.  A lane writes column r of rows .. + 4h, so rows four apart
// must not share banks: for W >= 64 the columns of every other group of four rows are XORed with 32
// (a row is a multiple of the 64 banks wide), the narrow W = 32 layout pads its rows instead.
template <int TN>
struct StageLayout {
  static constexpr int W = 32 * TN;
  static constexpr int PITCH = TN == 1 ? W + 8 : W;
  static __device__ __forceinline__ int at(int row, int col) {
    if constexpr (TN == 1) return row * PITCH + col;
    else return row * W + (col ^ (((row >> 2) & 1) << 5));
  }
};

// Vector path of one pass: RP rows x W columns starting at (row0, col0), every row and column in
// range and all accesses aligned, so that the loop is free of per-lane conditions.  Lane l handles
// four consecutive columns; the LDS reads and the dependent global reads (old C, aux) of U row
// segments are in flight together.
// CS: the lane also adds what it stores to cs[0..3], the running sums of its four columns.
// UMAX bounds the row segments in flight per lane (the eight-wave kernel has half the registers per wave).
template <int EPI, bool CB, bool BETA, int TN, int RP, bool CS = false, int UMAX = 4>
__device__ __forceinline__ void epilogue_pass_vec(const GemmArgs &g, const float *stage, int row0, int col0, int lane, float *cs = nullptr) {
  using L = StageLayout<TN>;
  constexpr int CPR = L::W / 4, RPI = 64 / CPR;            // 16-byte chunks per row, rows per wave-wide access
  constexpr int NIT = RP / RPI, U0 = NIT >= 8 ? 4 : NIT / 2, U = U0 < UMAX ? U0 : UMAX;
  constexpr bool kAux = EPI == CHN_EPI_RELU_BWD || EPI == CHN_EPI_GELU_BWD;
  // a lane keeps its four columns for the whole pass and walks down the rows
  const int cl = (lane % CPR) * 4, col = col0 + cl, rl0 = lane / CPR;
  Vec4 bias;
#pragma unroll
  for (int e = 0; e < 4; ++e) bias.v[e] = 0.0f;
  if constexpr (EPI >= CHN_EPI_BIAS && EPI <= CHN_EPI_BIAS_GELU) bias = load4v(g.bias, col, 0);
  // The global reads of the next batch are issued before the current one is worked on, so that only
  // the first batch's memory latency is exposed (a wave has its SIMD to itself here: nobody else would
  // hide it).
  auto fetch = [&](EpiRaw<CB> (&in)[U], int base) __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = row0 + rl0 + (base + u) * RPI;
      if constexpr (BETA) in[u].c0 = load4raw<CB>(g.C, (int64_t)row * g.ldc + col);
      if constexpr (kAux) in[u].aux = load4raw<CB>(g.aux, (int64_t)row * g.ldaux + col);
    }
  };
  auto compute = [&](const EpiRaw<CB> (&in)[U], int base) __attribute__((always_inline)) {
    f32x4 a[U];
#pragma unroll
    for (int u = 0; u < U; ++u) a[u] = *reinterpret_cast<const f32x4 *>(stage + L::at(rl0 + (base + u) * RPI, cl));
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if constexpr (CS) {
        Vec4 st;
        finish4_t<EPI, CB, BETA>(g, row0 + rl0 + (base + u) * RPI, col, a[u], in[u], bias, &st);
#pragma unroll
        for (int e = 0; e < 4; ++e) cs[e] += st.v[e];
      } else {
        finish4_t<EPI, CB, BETA>(g, row0 + rl0 + (base + u) * RPI, col, a[u], in[u], bias);
      }
    }
  };
  // Two register sets take turns (the last iteration fetches its own batch once more rather than
  // branch); the scheduling fences keep the compiler from moving the reads back next to their use.
  static_assert(NIT % (2 * U) == 0, "batches come in pairs");
  EpiRaw<CB> ea[U], eb[U];
  fetch(ea, 0);
#pragma unroll 1
  for (int base = 0; base < NIT; base += 2 * U) {
    fetch(eb, base + U);
    __builtin_amdgcn_sched_barrier(0);
    compute(ea, base);
    __builtin_amdgcn_sched_barrier(0);
    fetch(ea, min(base + 2 * U, NIT - U));
    __builtin_amdgcn_sched_barrier(0);
    compute(eb, base + U);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// One pass of a wave's epilogue: RP rows x W columns of staged accumulators.  With K splits the raw
// sums go to this split's slab of the workspace instead.
template <int TN, int RP, int UMAX = 4>
__device__ __forceinline__ void epilogue_pass(const GemmArgs &g, const float *stage, int row0, int col0, int lane, float *slab, float *cs) {
  using L = StageLayout<TN>;
  constexpr int W = L::W, CPR = W / 4;
  if (slab) {                                                 // split-K: raw sums, always aligned (ldp % 4 == 0)
#pragma unroll 1
    for (int c = lane; c < RP * CPR; c += 64) {
      const int rl = c / CPR, cl = (c % CPR) * 4;
      if (row0 + rl < g.M && col0 + cl < g.N)
        global_store<f32x4>(reinterpret_cast<uintptr_t>(slab + (int64_t)(row0 + rl) * g.ldp + col0 + cl),
                            *reinterpret_cast<const f32x4 *>(stage + L::at(rl, cl)));
    }
  } else if (g.epi_vec && col0 + W <= g.N && row0 + RP <= g.M) {
    auto run = [&](auto epi_c) __attribute__((always_inline)) {
      constexpr int EPI = decltype(epi_c)::value;
      constexpr bool kF32Only = EPI == CHN_EPI_BF16_COPY;   // (the host refuses a bf16 C for it)
      if constexpr (EPI == CHN_EPI_RELU_BWD || EPI == CHN_EPI_GELU_BWD) {
        if (g.colsum) {                                     // (the host asks for column sums with beta = 0 only)
          if (g.c_bf16) epilogue_pass_vec<EPI, true, false, TN, RP, true, UMAX>(g, stage, row0, col0, lane, cs);
          else epilogue_pass_vec<EPI, false, false, TN, RP, true, UMAX>(g, stage, row0, col0, lane, cs);
          return;
        }
      }
      if (g.beta != 0.0f) {
        if (!kF32Only && g.c_bf16) epilogue_pass_vec<EPI, !kF32Only, true, TN, RP, false, UMAX>(g, stage, row0, col0, lane);
        else epilogue_pass_vec<EPI, false, true, TN, RP, false, UMAX>(g, stage, row0, col0, lane);
      } else {
        if (!kF32Only && g.c_bf16) epilogue_pass_vec<EPI, !kF32Only, false, TN, RP, false, UMAX>(g, stage, row0, col0, lane);
        else epilogue_pass_vec<EPI, false, false, TN, RP, false, UMAX>(g, stage, row0, col0, lane);
      }
    };
    switch (g.epi) {
      case CHN_EPI_NONE: run(std::integral_constant<int, CHN_EPI_NONE>{}); break;
      case CHN_EPI_BIAS: run(std::integral_constant<int, CHN_EPI_BIAS>{}); break;
      case CHN_EPI_BIAS_RELU: run(std::integral_constant<int, CHN_EPI_BIAS_RELU>{}); break;
      case CHN_EPI_BIAS_GELU: run(std::integral_constant<int, CHN_EPI_BIAS_GELU>{}); break;
      case CHN_EPI_RELU_BWD: run(std::integral_constant<int, CHN_EPI_RELU_BWD>{}); break;
      case CHN_EPI_GELU_BWD: run(std::integral_constant<int, CHN_EPI_GELU_BWD>{}); break;
      default: run(std::integral_constant<int, CHN_EPI_BF16_COPY>{}); break;
    }
  } else if (g.epi_vec) {                                     // edge tile of aligned operands: whole 4-column groups that lie in range
    // (the lanes are dealt out over the groups that exist, so the number of dependent iterations
    // follows the part of the pass that is in range)
    const int nr = max(0, min(RP, g.M - row0)), ncg = max(0, min(CPR, (g.N - col0 + 3) >> 2));   // (a pass may lie wholly outside)
#pragma unroll 1
    for (int c = lane; c < nr * ncg; c += 64) {
      const int rl = c / ncg, cl = (c - rl * ncg) * 4, row = row0 + rl, col = col0 + cl;
      if (col + 4 <= g.N) {
        finish4(g, row, col, *reinterpret_cast<const f32x4 *>(stage + L::at(rl, cl)), epi_fetch(g, row, col));
      } else {
        for (int e = 0; col + e < g.N; ++e) finish1(g, row, col + e, stage[L::at(rl, cl + e)]);
      }
    }
  } else {                                                    // unaligned views: one element at a time
#pragma unroll 1
    for (int c = lane; c < RP * W; c += 64) {
      const int rl = c / W, cl = c % W;
      if (row0 + rl < g.M && col0 + cl < g.N) finish1(g, row0 + rl, col0 + cl, stage[L::at(rl, cl)]);
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
  // slabs are read eight at a time (all loads of a batch in flight together; slabs past the last one
  // read zeros) and added in split order, so the sum does not depend on the batching
  const uintptr_t zero = reinterpret_cast<uintptr_t>(&kZeroChunk);
  f32x4 a = global_load<f32x4>(reinterpret_cast<uintptr_t>(p));
  for (int s0 = 1; s0 < g.splits; s0 += 8) {
    f32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = global_load<f32x4>(s0 + u < g.splits ? reinterpret_cast<uintptr_t>(p + (s0 + u) * slab) : zero);
#pragma unroll
    for (int u = 0; u < 8; ++u) a += v[u];
  }
  if (g.epi_vec && col + 4 <= g.N) {
    finish4(g, row, col, a, epi_fetch(g, row, col));
  } else {
    for (int e = 0; e < 4 && col + e < g.N; ++e) finish1(g, row, col + e, a[e]);
  }
}

// Which C tile (and which K split) a workgroup owns: XCD-aware renumbering, then grouped (8 tile rows
// at a time) ordering.
struct TilePos { int tm, tn, split; };
__device__ __forceinline__ TilePos tile_pos(const GemmArgs &g) {
  const int nb = g.tiles_m * g.tiles_n;
  int pid = blockIdx.x % nb;
  const int split = blockIdx.x / nb;
  const int nb8 = nb & ~7;
  if (pid < nb8) pid = (pid & 7) * (nb8 >> 3) + (pid >> 3);
  constexpr int GROUP = 8;
  const int width = GROUP * g.tiles_n;
  const int first_m = (pid / width) * GROUP;
  const int gsize = min(g.tiles_m - first_m, GROUP);
  return TilePos{first_m + (pid % width) % gsize, (pid % width) / gsize, split};
}

// Epilogue of one workgroup.  Each wave moves its accumulators through its own LDS area `stage`
// (kEpiStageBytes<TM, TN> bytes; the caller has made sure that nobody uses that memory for anything
// else any more) in passes of up to 64 rows: MFMA layout in, row-major out, so that bias / activation
// / activation-gradient run on 16-byte vectors and C, aux and preact are touched as whole row
// segments.  A lane holds, per 32x32 block, column r and rows 8*(v/4) + 4*h + v%4.  Only the
// register-to-LDS part exists once per pass (accumulator registers cannot be indexed at run time);
// everything after it is one loop, so the code a wave runs through stays small.
template <int TM, int TN>
constexpr int kEpiRows = TM == 1 ? 32 : 64;
template <int TM, int TN>
constexpr int kEpiStageBytes = kEpiRows<TM, TN> * StageLayout<TN>::PITCH * 4;

// WAVES_N: waves side by side along N (2 for the 2 x 2 arrangement of four waves, 4 for the 2 x 4 of eight).
template <int TM, int TN, int WAVES_N = 2>
__device__ __forceinline__ void write_out(const GemmArgs &g, floatx16 (&acc)[TM][TN], char *stage_bytes, int m0, int n0, int split) {
  using L = StageLayout<TN>;
  constexpr int RP = kEpiRows<TM, TN>, IPP = RP / 32, NPASS = TM / IPP;   // 32-row blocks per pass, passes
  // (the lane id is taken from the hardware rather than from threadIdx.x: otherwise the compiler keeps
  // the value computed before the K loop alive across it, in a kernel that has no register to spare)
  const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  const int lane = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int r = lane & 31, h = lane >> 5;
  float *stage = reinterpret_cast<float *>(stage_bytes);
  float *slab = g.splits > 1 ? g.partial + (int64_t)split * g.M * g.ldp : nullptr;
  auto put = [&](auto pc) {
    constexpr int P = decltype(pc)::value;
#pragma unroll
    for (int ii = 0; ii < IPP; ++ii)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
#pragma unroll
        for (int v = 0; v < 16; ++v)
          stage[L::at(ii * 32 + 8 * (v >> 2) + 4 * h + (v & 3), j * 32 + r)] = acc[P * IPP + ii][j][v];
        __builtin_amdgcn_sched_barrier(0);   // one block's 16 values in flight at a time, not the whole pass
      }
  };
  float cs[4] = {0.0f, 0.0f, 0.0f, 0.0f};               // column sums of this wave's rows (when asked for)
#pragma unroll 1
  for (int p = 0; p < NPASS; ++p) {
    if (p == 0) put(std::integral_constant<int, 0>{});
    else put(std::integral_constant<int, NPASS - 1>{});
    __builtin_amdgcn_wave_barrier();
    epilogue_pass<TN, RP, WAVES_N == 4 ? 2 : 4>(g, stage, m0 + (wm * TM) * 32 + p * RP, n0 + wn * TN * 32, lane, slab, cs);
    __builtin_amdgcn_wave_barrier();
  }
  if constexpr (TM == 4 && (TN == 4 || TN == 2)) {
    // The lanes of one row segment own 8 * TN column groups; lanes that differ by a multiple of that
    // walked different rows of the same columns.  One row of the sums per wave tile (128 rows of C).
    if (g.colsum) {
      constexpr int CPR = 8 * TN;
      f32x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float t = cs[e];
#pragma unroll
        for (int o = 32; o >= CPR; o >>= 1) t += __shfl_xor(t, o, 64);
        v[e] = t;
      }
      if (lane < CPR)
        global_store<f32x4>(reinterpret_cast<uintptr_t>(g.colsum + (int64_t)((m0 >> 7) + wm) * g.ldcs + n0 + wn * (32 * TN) + lane * 4), v);
    }
  }
}

// PB / PB2: bytes per global load piece of A / of B
template <typename T, int TM, int TN, bool A_KC, bool B_KC, int PB, int PB2 = PB>
__global__ __launch_bounds__(256) void gemm_kernel(GemmArgs g) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  constexpr int BK = 128 / sizeof(T);               // elements of k per tile step
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
  extern __shared__ __align__(16) char lds[];

  const TilePos tp = tile_pos(g);
  const int split = tp.split, m0 = tp.tm * BM, n0 = tp.tn * BN;

  TileLoader<T, BM, A_KC, PB> la;
  TileLoader<T, BN, B_KC, PB2> lb;
  la.init(static_cast<const T *>(g.A), g.lda, g.M, m0, g.K);
  lb.init(static_cast<const T *>(g.B), g.ldb, g.N, n0, g.K, 128);

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

  // The small tiles look two tiles ahead: with few MFMAs per tile step, the two k-steps between the
  // issue of a tile's loads and their move to LDS do not cover a trip to memory, and a workgroup that
  // is alone on its compute unit (small products) then runs at one memory latency per tile step.  Two
  // sets of staging registers take turns, the loop is written out for both so that each set is named
  // at compile time: a tile's loads are issued right after the set has been emptied, a whole tile step
  // before they are needed.
  constexpr bool kDeep = TM * TN <= 4;
  if constexpr (kDeep) {
    la.template issue<0>((kt0 + 1) * BK);
    lb.template issue<0>((kt0 + 1) * BK);
    la.template issue<1>((kt0 + 2) * BK);
    lb.template issue<1>((kt0 + 2) * BK);
    auto step = [&](auto set_c, int kt) __attribute__((always_inline)) {
      constexpr int SET = decltype(set_c)::value;
      const char *cur = lds + ((kt - kt0) & 1) * STAGE;
      char *nxt = lds + ((kt - kt0 + 1) & 1) * STAGE;
      f1.read(cur + a_row, cur + b_row, koff[1]);
      mma<T, TM, TN>(acc, f0);
      f0.read(cur + a_row, cur + b_row, koff[2]);
      mma<T, TM, TN>(acc, f1);
      f1.read(cur + a_row, cur + b_row, koff[3]);
      la.template store<SET>(nxt);                    // tile kt + 1, on its way since the step before
      lb.template store<SET>(nxt + A_BYTES);
      la.template issue<SET>((kt + 3) * BK);          // (past the end of K: zeros, never used)
      lb.template issue<SET>((kt + 3) * BK);
      mma<T, TM, TN>(acc, f0);
      __syncthreads();
      f0.read(nxt + a_row, nxt + b_row, koff[0]);
      mma<T, TM, TN>(acc, f1);
    };
    int kt = kt0;
    for (; kt + 1 < nk; kt += 2) {
      step(std::integral_constant<int, 0>{}, kt);
      step(std::integral_constant<int, 1>{}, kt + 1);
    }
    if (kt < nk) step(std::integral_constant<int, 0>{}, kt);
  } else
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

  __syncthreads();   // every wave is done with the operand stages
  write_out<TM, TN>(g, acc, lds + (threadIdx.x >> 6) * kEpiStageBytes<TM, TN>, m0, n0, split);
}

// ---- big tile, K-contiguous operands copied by the memory pipeline itself ---------------------------
// A K-contiguous operand tile needs no arithmetic on its way into LDS, so gfx950's 16-byte
// global-load-to-LDS instruction can move it: no staging registers, no LDS store instructions, and
// the copy may be in flight for a whole tile step.  One such instruction writes the 64 lanes' chunks
// to 1024 consecutive LDS bytes (8 tile rows), so the swizzle is applied on the global side: the
// lane that fills physical slot (row p, chunk c) fetches the logical chunk that lives there.
template <typename T, int ROWS, bool RAGGED, int NW = 4>
struct DmaLoader {
  static constexpr int EPC = Traits<T>::EPC;
  static constexpr int BK = 128 / (int)sizeof(T);
  static constexpr int NS = ROWS / (8 * NW);   // instructions per wave and tile (NW waves share the tile)
  const char *tile;                        // wave-uniform: first row of the tile, k = 0
  uint32_t off[NS];                        // byte offset of the slot's chunk from `tile`
  int lim[RAGGED ? NS : 1];                // RAGGED: K - (k offset of the slot's chunk)
  int wave, k_last;                        // wave-uniform

  // K is a multiple of the chunk length (16-byte pieces), so a chunk is never partly valid along k.
  // Without RAGGED, K is also a multiple of BK and every chunk of every tile exists; with it, chunks at
  // or past K are fetched from the zero chunk.  Rows past the operand's end are read from its last row
  // instead: they only feed rows or columns of C that are never written.
  __device__ __forceinline__ void init(const T *base, int64_t ld, int rows_total, int row0, int K) {
    wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    k_last = K - BK;
    tile = reinterpret_cast<const char *>(base + (int64_t)row0 * ld);
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < NS; ++i) {
      const int slot = (i * NW + wave) * 64 + lane;
      const int prow = slot >> 3, pchunk = slot & 7;
      const int row = lds_row<T>(prow);                 // the row swap is its own inverse
      const int kc = (pchunk ^ ((row >> 1) & 7)) * EPC;
      const int rowc = min(row, rows_total - 1 - row0);
      off[i] = (uint32_t)(((int64_t)rowc * ld + kc) * (int64_t)sizeof(T));
      if constexpr (RAGGED) lim[i] = K - kc;
    }
  }

  // Start the copy of the tile whose first k is k0 into the operand's part of a stage.  Tiles past
  // the end of K (requested by the last steps, never used) re-read the last tile or read zeros.
  template <int FIRST = 0, int COUNT = NS>
  __device__ __forceinline__ void issue(int k0, char *lds_operand) const {
    const char *p = tile + (int64_t)(RAGGED ? k0 : min(k0, k_last)) * (int64_t)sizeof(T);
    const char *zero = reinterpret_cast<const char *>(&kZeroChunk);
#pragma unroll
    for (int i = FIRST; i < FIRST + COUNT; ++i) {
      const char *a = p + off[i];
      if constexpr (RAGGED) a = k0 < lim[i] ? a : zero;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)a,
                                       (__attribute__((address_space(3))) void *)(lds_operand + (i * NW + wave) * 1024),
                                       16, 0, 0);
    }
  }
};

// The same for a bf16 operand whose unit stride runs along M/N: the tile goes to LDS as it lies in
// memory, BK rows of k, each ROWS elements (512 bytes) of m, and is transposed on the way out of LDS
// by the 16-bit transposing read (see TrReader).  The eight 64-byte blocks of a k-row are XORed with
// k % 8, so that the four k-rows one group of lanes reads together sit in different banks.
template <int ROWS, bool RAGGED, int NW = 4>
struct DmaLoaderMC {
  static_assert(ROWS == 256, "one k-row must be 512 bytes");
  static constexpr int BK = 64, NS = BK * 512 / 1024 / NW;   // instructions per wave and tile
  const char *tile;                        // wave-uniform: element (k = 0, m = row0)
  uint32_t off[NS];
  int lim[RAGGED ? NS : 1];                // RAGGED: K - (k-row of the slot)
  int wave, k_last;
  int64_t kbytes;                          // bytes between consecutive k

  // rows_total is a multiple of 8 (16-byte pieces); chunks past it re-read the operand's last chunk
  // and only feed rows or columns of C that are never written.
  __device__ __forceinline__ void init(const bf16_raw *base, int64_t ld, int rows_total, int row0, int K) {
    wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    k_last = K - BK;
    kbytes = ld * 2;
    tile = reinterpret_cast<const char *>(base + row0);
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < NS; ++i) {
      const int slot = (i * NW + wave) * 64 + lane;
      const int k = slot >> 5, p = slot & 31;                  // k-row, 16-byte slot inside it
      const int m = (((p >> 2) ^ (k & 7)) * 32) + (p & 3) * 8; // the 8 elements that live in that slot
      const int mc = min(m, rows_total - 8 - row0);
      off[i] = (uint32_t)(((int64_t)k * ld + mc) * 2);
      if constexpr (RAGGED) lim[i] = K - k;
    }
  }

  template <int FIRST = 0, int COUNT = NS>
  __device__ __forceinline__ void issue(int k0, char *lds_operand) const {
    const char *p = tile + (int64_t)(RAGGED ? k0 : min(k0, k_last)) * kbytes;
    const char *zero = reinterpret_cast<const char *>(&kZeroChunk);
#pragma unroll
    for (int i = FIRST; i < FIRST + COUNT; ++i) {
      const char *a = p + off[i];
      if constexpr (RAGGED) a = k0 < lim[i] ? a : zero;   // k-rows at or past K read as zeros
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)a,
                                       (__attribute__((address_space(3))) void *)(lds_operand + (i * NW + wave) * 1024),
                                       16, 0, 0);
    }
  }
};

// Fragment readers of the direct-copy kernel: read(stage, k-step, 32-row block)
// returns the lane's 16 bytes (8 bf16 or 4 fp32 along k) for an MFMA.
// K-packed tile (lds_off layout): one 16-byte read.
template <typename T>
struct KcReader {
  int row, koff[4];
  // first_block: the wave's first 32-row block; region: byte offset of the operand's part of a stage
  __device__ __forceinline__ void init(int first_block, int lane, int region) {
    const int r = lane & 31, h = lane >> 5;
    row = region + (first_block * 32 + lds_row<T>(r)) * 128;
    const int sw = (r >> 1) & 7;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) koff[ks] = ((ks * 2 + h) ^ sw) << 4;
  }
  __device__ __forceinline__ uint4 read(const char *stage, int ks, int i) const {
    return *reinterpret_cast<const uint4 *>(stage + row + i * (32 * 128) + koff[ks]);
  }
};
// bf16 tile stored [k][m] (DmaLoaderMC): two transposing 8-byte reads.  Within a group of 16 lanes the
// instruction hands lane i element (i % 4) of the 8 bytes addressed by lanes i/4, 4 + i/4, 8 + i/4 and
// 12 + i/4; so lane 4e + q of a group points at (k = .. + e, m = .. + 4q), and every lane ends up with
// four consecutive k of its own m.  Lanes 0-31 / 32-63 take k 0-7 / 8-15 of the k-step like the K-packed
// reader, first read k .. + 0-3, second read k .. + 4-7.
typedef short short4v __attribute__((ext_vector_type(4)));
struct TrReader {
  int base[4][2];   // per 32-row block and half: byte offset inside a stage, k-step 0
  __device__ __forceinline__ void init(int first_block, int lane, int region) {
    const int G = lane >> 4, s = lane & 15, e = s >> 2, q = s & 3, h = G >> 1, g1 = G & 1;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const int k = 8 * h + 4 * t + e;
        base[i][t] = region + k * 512 + (((first_block + i) ^ (k & 7)) * 64) + (16 * g1 + 4 * q) * 2;
      }
  }
  __device__ __forceinline__ uint4 read(const char *stage, int ks, int i) const {
    typedef __attribute__((address_space(3))) short4v *lds_ptr;
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(stage + base[i][0] + ks * (16 * 512)));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(stage + base[i][1] + ks * (16 * 512)));
    const uint2 l = __builtin_bit_cast(uint2, lo), u = __builtin_bit_cast(uint2, hi);
    return make_uint4(l.x, l.y, u.x, u.y);
  }
};

// Pull the cache lines of a BM x BN tile of a row-major array (C or aux, `esz` bytes per element)
// towards L2 without spending registers or branches: four bytes of every line are copied to a scrap
// area in LDS.  `scrap` needs 1024 bytes; nothing ever reads it.
template <int BM, int BN>
__device__ __forceinline__ void touch_tile(const void *p, int64_t ld, int esz, int M, int N, int m0, int n0, char *scrap) {
  const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  constexpr int SEG = 8, NT = BM * SEG / 256;     // eight touches per row: every 128 (fp32) or 64 (bf16) bytes
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int i = threadIdx.x + t * 256;
    const int row = min(m0 + i / SEG, M - 1);
    const int col = min(n0 + (i % SEG) * (BN / SEG), N - 1) & ~1;
    const char *a = static_cast<const char *>(p) + ((int64_t)row * ld + col) * esz;
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)a,
                                     (__attribute__((address_space(3))) void *)(scrap + wave * 256), 4, 0, 0);
  }
}

// 256 x 256 tile with at least one K-contiguous operand whose rows allow 16-byte pieces.  The two
// stages are two separate LDS arrays and the K loop is written out for both roles of them: only
// then can the compiler tell that a copy in flight into one stage does not concern the fragment
// reads of the other, and leave the wait for the copy to the barrier.
// One tile step: k-steps 0..2 out of `cur` while the copy of the next tile (started one step ago)
// lands in `nxt`; barrier (copy complete, nobody reads `cur` any more); start the copy of the tile
// after the next into `cur`; k-step 3 while the first fragments of `nxt` are read.
template <typename T, bool A_KC, bool B_KC, bool RAGGED>
__global__ __launch_bounds__(256) void gemm_kernel_dma(GemmArgs g) {
  // How each operand reaches LDS: K-contiguous -> direct copy, K-packed; bf16 M/N-contiguous -> direct
  // copy as it lies, transposing reads; fp32 M/N-contiguous -> through registers (TileLoader).
  constexpr bool kBf16 = sizeof(T) == 2;
  constexpr bool A_DMA = A_KC || kBf16, B_DMA = B_KC || kBf16;
  static_assert(A_DMA || B_DMA, "at least one operand must be copied directly");
  constexpr int TM = 4, TN = 4, BM = 256, BN = 256;
  constexpr int BK = 128 / sizeof(T);
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
  // (each stage is followed by 1 KB of scrap for touch_tile: as part of the same array it falls into
  // the same class as the stage's real copies when the compiler decides which LDS reads must wait)
  __shared__ __align__(1024) char stage0[STAGE + 1024];
  __shared__ __align__(1024) char stage1[STAGE + 1024];

  const TilePos tp = tile_pos(g);
  const int split = tp.split, m0 = tp.tm * BM, n0 = tp.tn * BN;

  std::conditional_t<A_KC, DmaLoader<T, BM, RAGGED>, std::conditional_t<kBf16, DmaLoaderMC<BM, RAGGED>, TileLoader<T, BM, false, 16>>> la;
  std::conditional_t<B_KC, DmaLoader<T, BN, RAGGED>, std::conditional_t<kBf16, DmaLoaderMC<BN, RAGGED>, TileLoader<T, BN, false, 16>>> lb;
  la.init(static_cast<const T *>(g.A), g.lda, g.M, m0, g.K);
  lb.init(static_cast<const T *>(g.B), g.ldb, g.N, n0, g.K);

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const int r = lane & 31, h = lane >> 5;

  std::conditional_t<A_KC || !kBf16, KcReader<T>, TrReader> ra;
  std::conditional_t<B_KC || !kBf16, KcReader<T>, TrReader> rb;
  ra.init(wm * TM, lane, 0);
  rb.init(wn * TN, lane, A_BYTES);
  auto read_frags = [&](Frags<TM, TN> &f, const char *stage, int ks) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < TM; ++i) f.a[i] = ra.read(stage, ks, i);
#pragma unroll
    for (int j = 0; j < TN; ++j) f.b[j] = rb.read(stage, ks, j);
  };

  const int nk_all = (g.K + BK - 1) / BK;
  const int per_split = (nk_all + g.splits - 1) / g.splits;
  const int kt0 = split * per_split;
  const int nk = min(nk_all, kt0 + per_split);

  auto k_of = [&](int kt) { return kt * BK; };   // first k of tile step kt

  // prologue: first tile into stage 0, second tile on its way into stage 1
  if constexpr (A_DMA) { la.issue(k_of(kt0), stage0); la.issue(k_of(kt0 + 1), stage1); }
  else { la.issue(k_of(kt0)); la.store(stage0); }
  if constexpr (B_DMA) {
    lb.issue(k_of(kt0), stage0 + A_BYTES);
    if constexpr (!(A_DMA && B_DMA)) lb.issue(k_of(kt0 + 1), stage1 + A_BYTES);   // (else: in the first step's k-step 0)
  } else { lb.issue(k_of(kt0)); lb.store(stage0 + A_BYTES); }
  // (the accumulators are cleared while the first copies are in flight)
  __builtin_amdgcn_sched_barrier(0);
  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
  __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
  __syncthreads();
  Frags<TM, TN> f0, f1;
  read_frags(f0, stage0, 0);

  constexpr int NM = (sizeof(T) == 2 ? 1 : 4) * TM * TN;   // MFMAs per k-step
  constexpr int NG = TM + TN;                              // fragments (scheduling groups) per k-step
  constexpr int RPG_A = (A_KC || !kBf16) ? 1 : 2, RPG_B = (B_KC || !kBf16) ? 1 : 2;   // LDS reads per fragment
  constexpr int NMC = (A_DMA ? 0 : 8) + (B_DMA ? 0 : 8);   // 16-byte register loads per step (fp32 transposed operand)
  constexpr int NDMA = (A_DMA ? 8 : 0) + (B_DMA ? 8 : 0);  // direct copies per wave and step
  // interleaving hint for one k-step: per fragment its LDS reads, then `vm` memory instructions of
  // class `vmask`, then its share of the MFMAs
  auto sched_kstep = [&](auto vmask_c, auto vm_c) __attribute__((always_inline)) {
    constexpr int vmask = decltype(vmask_c)::value, vm = decltype(vm_c)::value;
#pragma unroll
    for (int s = 0; s < TM; ++s) {
      __builtin_amdgcn_sched_group_barrier(SG_DS_READ, RPG_A, 0);
      if constexpr (vm > 0) __builtin_amdgcn_sched_group_barrier(vmask, vm, 0);
      __builtin_amdgcn_sched_group_barrier(SG_MFMA, NM / NG, 0);
    }
#pragma unroll
    for (int s = 0; s < TN; ++s) {
      __builtin_amdgcn_sched_group_barrier(SG_DS_READ, RPG_B, 0);
      if constexpr (vm > 0) __builtin_amdgcn_sched_group_barrier(vmask, vm, 0);
      __builtin_amdgcn_sched_group_barrier(SG_MFMA, NM / NG, 0);
    }
  };
  using IC0 = std::integral_constant<int, 0>;

  // B's copy runs half a step behind A's when both are direct (SPLIT): the copy instructions of a tile
  // are then spread over two k-steps instead of crowding the MFMAs of one.
  constexpr bool SPLIT = A_DMA && B_DMA;
  auto step = [&](char *cur, char *nxt, int kt) __attribute__((always_inline)) {
    // k-step 0 (an fp32 transposed operand's loads of the next tile are issued here and written in
    // k-step 2; with SPLIT, B's copy of the next tile starts here: `nxt` has been free since the
    // previous step's barrier)
    read_frags(f1, cur, 1);
    if constexpr (!A_DMA) la.issue(k_of(kt + 1));
    if constexpr (!B_DMA) lb.issue(k_of(kt + 1));
    if constexpr (SPLIT) lb.issue(k_of(kt + 1), nxt + A_BYTES);
    mma<T, TM, TN>(acc, f0);
    if constexpr (SPLIT) sched_kstep(std::integral_constant<int, SG_VMEM>{}, std::integral_constant<int, 8 / NG>{});
    else sched_kstep(std::integral_constant<int, SG_VMEM_READ>{}, std::integral_constant<int, NMC / NG>{});
    // k-step 1
    read_frags(f0, cur, 2);
    mma<T, TM, TN>(acc, f1);
    sched_kstep(IC0{}, IC0{});
    // k-step 2
    read_frags(f1, cur, 3);
    mma<T, TM, TN>(acc, f0);
    sched_kstep(IC0{}, IC0{});
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (!A_DMA) la.store(nxt);
    if constexpr (!B_DMA) lb.store(nxt + A_BYTES);
    // A wave's own copies must have landed before it tells the others so: the counter of the vector
    // memory pipeline (which also tracks copies to LDS) has to be zero ahead of the barrier.
    __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
    // k-step 3, overlapped with the first fragment reads of the next stage and with the issue of the
    // copies of the tile after the next (their target, `cur`, is free from here on)
    if constexpr (A_DMA) la.issue(k_of(kt + 2), cur);
    if constexpr (B_DMA && !SPLIT) lb.issue(k_of(kt + 2), cur + A_BYTES);
    read_frags(f0, nxt, 0);
    mma<T, TM, TN>(acc, f1);
    sched_kstep(std::integral_constant<int, SG_VMEM>{}, std::integral_constant<int, (SPLIT ? 8 : NDMA) / NG>{});
    __builtin_amdgcn_sched_barrier(0);
  };

  int kt = kt0;
  for (; kt + 3 < nk; kt += 2) {
    step(stage0, stage1, kt);
    step(stage1, stage0, kt + 1);
  }
  // Two or three steps to go.  The epilogue's own reads (old C, retained activation) would each cost
  // a trip to HBM with nobody to hide it, so their lines are requested now and wait in L2.  (Outside
  // the main loop on purpose: with these extra copies around, the compiler makes the fragment reads
  // of the following step wait for all copies in flight.  They go to the scrap of stage 1, the stage
  // the next step does not read before its barrier.)
  if (g.splits == 1) {
    const int esz = g.c_bf16 ? 2 : 4;
    if (g.beta != 0.0f) touch_tile<BM, BN>(g.C, g.ldc, esz, g.M, g.N, m0, n0, stage1 + STAGE);
    if (g.epi == CHN_EPI_RELU_BWD || g.epi == CHN_EPI_GELU_BWD) touch_tile<BM, BN>(g.aux, g.ldaux, esz, g.M, g.N, m0, n0, stage1 + STAGE);
  }
  for (; kt + 1 < nk; kt += 2) {
    step(stage0, stage1, kt);
    step(stage1, stage0, kt + 1);
  }
  if (kt < nk) step(stage0, stage1, kt);

  // The (unused) copies that the last steps started must be over: the epilogue reuses stage 0.
  __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
  __syncthreads();
  static_assert(2 * kEpiStageBytes<TM, TN> <= STAGE, "two waves stage their accumulators in each operand stage");
  write_out<TM, TN>(g, acc, (wave < 2 ? stage0 : stage1) + (wave & 1) * kEpiStageBytes<TM, TN>, m0, n0, split);
}

// ---- 256 x 256 tile, eight waves ----------------------------------------------------------------------
// The loaders of the four-wave kernel with their instructions in two parts (first and second half), so that
// a tile's copies can be dealt out over several k-steps.
template <typename L>
struct TwoParts : L {
  template <int P>
  __device__ __forceinline__ void issue_part(int k0, char *lds_operand) const {
    this->template issue<P * (L::NS / 2), L::NS / 2>(k0, lds_operand);
  }
};

// bfloat16 only.  The tile of the direct-copy kernel above with the work dealt out to eight waves, two on
// every SIMD, in a 2 (M) x 4 (N) arrangement: a wave owns 128 x 64 of C (4 x 2 MFMA blocks, 128 accumulator
// registers), so that two waves fit the register file of a SIMD.  Whatever one wave waits for -- fragment
// reads, the barrier of a tile step, a copy instruction that the memory pipeline does not take yet, the
// staging and stores of its epilogue -- the other wave's MFMAs fill.
// Operand traffic from L2 is that of the four-wave kernel (the tile is the same), LDS fragment traffic is
// 1.5 times higher (6 fragment reads per 8 MFMAs instead of 8 per 16).
//
// BN = 128 is the same kernel on a 256 x 128 tile for products whose N is too small to give 256 workgroups
// of the square tile (a classifier's logits): the waves stand 4 (M) x 2 (N), a wave owns 64 x 64 (2 x 2
// MFMA blocks), 6 copy instructions per wave and tile instead of 8, as many fragment reads as MFMAs.
template <bool A_KC, bool B_KC, bool RAGGED, int BN = 256>
__global__ __launch_bounds__(512) void gemm_kernel_w8(GemmArgs g) {
  using T = bf16_raw;
  static_assert(BN == 256 || (BN == 128 && A_KC && B_KC), "the 256 x 128 tile exists for K-contiguous operands");
  constexpr int BM = 256, NW = 8, WN = BN == 256 ? 4 : 2, WM = NW / WN;   // waves along N and M
  constexpr int TM = BM / (32 * WM), TN = BN / (32 * WN);
  constexpr int BK = 64;
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
  __shared__ __align__(1024) char stage0[STAGE];
  __shared__ __align__(1024) char stage1[STAGE];

  const TilePos tp = tile_pos(g);
  const int split = tp.split, m0 = tp.tm * BM, n0 = tp.tn * BN;

  TwoParts<std::conditional_t<A_KC, DmaLoader<T, BM, RAGGED, NW>, DmaLoaderMC<BM, RAGGED, NW>>> la;
  TwoParts<std::conditional_t<B_KC, DmaLoader<T, BN, RAGGED, NW>, DmaLoaderMC<BN, RAGGED, NW>>> lb;
  la.init(static_cast<const T *>(g.A), g.lda, g.M, m0, g.K);
  lb.init(static_cast<const T *>(g.B), g.ldb, g.N, n0, g.K);

  const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int wm = wave / WN, wn = wave % WN;

  std::conditional_t<A_KC, KcReader<T>, TrReader> ra;
  std::conditional_t<B_KC, KcReader<T>, TrReader> rb;
  ra.init(wm * TM, lane, 0);
  rb.init(wn * TN, lane, A_BYTES);
  auto read_frags = [&](Frags<TM, TN> &f, const char *stage, int ks) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < TM; ++i) f.a[i] = ra.read(stage, ks, i);
#pragma unroll
    for (int j = 0; j < TN; ++j) f.b[j] = rb.read(stage, ks, j);
  };

  const int nk_all = (g.K + BK - 1) / BK;
  const int per_split = (nk_all + g.splits - 1) / g.splits;
  const int kt0 = split * per_split;
  const int nk = min(nk_all, kt0 + per_split);
  auto k_of = [&](int kt) { return kt * BK; };

  // prologue: first tile into stage 0; of the second tile the part that a step issues after its barrier
  la.template issue_part<0>(k_of(kt0), stage0);
  la.template issue_part<1>(k_of(kt0), stage0);
  lb.template issue_part<0>(k_of(kt0), stage0 + A_BYTES);
  lb.template issue_part<1>(k_of(kt0), stage0 + A_BYTES);
  la.template issue_part<0>(k_of(kt0 + 1), stage1);
  __builtin_amdgcn_sched_barrier(0);
  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
  __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
  __syncthreads();
  Frags<TM, TN> f0, f1;
  read_frags(f0, stage0, 0);

  // interleaving hint for one k-step: per fragment its LDS reads, then (for the first NV fragments) one copy
  // instruction, then its share of the 8 MFMAs (2, 2, 1, 1, 1, 1)
  constexpr int RPG_A = A_KC ? 1 : 2, RPG_B = B_KC ? 1 : 2;   // LDS reads per fragment
#define CHN_W8_GROUP(S, RPG, NMF, NV)                                           \
  __builtin_amdgcn_sched_group_barrier(SG_DS_READ, RPG, 0);                     \
  if constexpr ((NV) > (S)) __builtin_amdgcn_sched_group_barrier(SG_VMEM, 1, 0); \
  __builtin_amdgcn_sched_group_barrier(SG_MFMA, NMF, 0);
#define CHN_W8_KSTEP(NV)                                                        \
  if constexpr (TM == 4) {                                                      \
    CHN_W8_GROUP(0, RPG_A, 2, NV) CHN_W8_GROUP(1, RPG_A, 2, NV) CHN_W8_GROUP(2, RPG_A, 1, NV) \
    CHN_W8_GROUP(3, RPG_A, 1, NV) CHN_W8_GROUP(4, RPG_B, 1, NV) CHN_W8_GROUP(5, RPG_B, 1, NV) \
  } else {                                                                      \
    CHN_W8_GROUP(0, RPG_A, 1, NV) CHN_W8_GROUP(1, RPG_A, 1, NV) CHN_W8_GROUP(2, RPG_B, 1, NV) \
    CHN_W8_GROUP(3, RPG_B, 1, NV)                                               \
  }

  // One tile step: k-steps 0..2 out of `cur` (the fragments of the following k-step are read while a
  // k-step multiplies); barrier -- the copy of the next tile has landed in `nxt`, and nobody reads `cur` any
  // more; k-step 3 multiplies out of registers while the first fragments of `nxt` are read.  The copies of
  // a tile are spread: A's first part right after the barrier that frees their stage (k-step 3), A's second
  // and B's first part in k-step 0 of the next step, B's second part in its k-step 1; they then have two
  // k-steps left to land, several times what a trip to L2 takes.
  auto step = [&](char *cur, char *nxt, int kt) __attribute__((always_inline)) {
    read_frags(f1, cur, 1);
    la.template issue_part<1>(k_of(kt + 1), nxt);
    lb.template issue_part<0>(k_of(kt + 1), nxt + A_BYTES);
    mma<T, TM, TN>(acc, f0);
    CHN_W8_KSTEP(BN == 256 ? 4 : 3)
    read_frags(f0, cur, 2);
    lb.template issue_part<1>(k_of(kt + 1), nxt + A_BYTES);
    mma<T, TM, TN>(acc, f1);
    CHN_W8_KSTEP(BN == 256 ? 2 : 1)
    read_frags(f1, cur, 3);
    mma<T, TM, TN>(acc, f0);
    CHN_W8_KSTEP(0)
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
    la.template issue_part<0>(k_of(kt + 2), cur);
    read_frags(f0, nxt, 0);
    mma<T, TM, TN>(acc, f1);
    CHN_W8_KSTEP(2)
    __builtin_amdgcn_sched_barrier(0);
  };
#undef CHN_W8_KSTEP
#undef CHN_W8_GROUP

  int kt = kt0;
  for (; kt + 1 < nk; kt += 2) {
    step(stage0, stage1, kt);
    step(stage1, stage0, kt + 1);
  }
  if (kt < nk) step(stage0, stage1, kt);

  // The (unused) copies that the last steps started must be over: the epilogue reuses both stages.
  __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
  __syncthreads();
  if constexpr (BN == 256) {
    static_assert(4 * kEpiStageBytes<TM, TN> <= STAGE, "four waves stage their accumulators in each operand stage");
    write_out<TM, TN, WN>(g, acc, (wave < 4 ? stage0 : stage1) + (wave & 3) * kEpiStageBytes<TM, TN>, m0, n0, split);
  } else {
    // three waves in each operand stage, two in an area of their own
    static_assert(3 * kEpiStageBytes<TM, TN> <= STAGE, "three waves stage their accumulators in each operand stage");
    __shared__ __align__(1024) char epi_extra[2 * kEpiStageBytes<TM, TN>];
    char *area = wave < 3 ? stage0 + wave * kEpiStageBytes<TM, TN>
               : wave < 6 ? stage1 + (wave - 3) * kEpiStageBytes<TM, TN> : epi_extra + (wave - 6) * kEpiStageBytes<TM, TN>;
    write_out<TM, TN, WN>(g, acc, area, m0, n0, split);
  }
}

template <bool A_KC, bool B_KC>
chn_status launch_w8(const GemmArgs &g, hipStream_t st) {
  const dim3 grid((unsigned)(g.tiles_m * g.tiles_n * g.splits));
  if (g.tile == 3) {
    if constexpr (A_KC && B_KC) {
      if (g.K % 64 == 0) hipLaunchKernelGGL((gemm_kernel_w8<true, true, false, 128>), grid, dim3(512), 0, st, g);
      else hipLaunchKernelGGL((gemm_kernel_w8<true, true, true, 128>), grid, dim3(512), 0, st, g);
    } else {
      return fail(CHN_ERR_LAUNCH, "gemm: the 256 x 128 tile was planned for operands it does not take");
    }
  } else if (g.K % 64 == 0) hipLaunchKernelGGL((gemm_kernel_w8<A_KC, B_KC, false>), grid, dim3(512), 0, st, g);
  else hipLaunchKernelGGL((gemm_kernel_w8<A_KC, B_KC, true>), grid, dim3(512), 0, st, g);
  CHN_TRY(check_launch("gemm (eight waves)"));
  if (g.splits > 1) {
    const int64_t n = (int64_t)g.M * (g.ldp / 4);
    hipLaunchKernelGGL(gemm_splitk_finish_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, g);
    return check_launch("gemm split-K finish");
  }
  return CHN_OK;
}

template <typename T, bool A_KC, bool B_KC>
constexpr bool kHasDmaKernel = A_KC || B_KC || sizeof(T) == 2;

template <typename T, bool A_KC, bool B_KC>
chn_status launch_dma(const GemmArgs &g, hipStream_t st) {
  if constexpr (kHasDmaKernel<T, A_KC, B_KC>) {
    const dim3 grid((unsigned)(g.tiles_m * g.tiles_n * g.splits));
    if (g.K % (128 / (int)sizeof(T)) == 0) hipLaunchKernelGGL((gemm_kernel_dma<T, A_KC, B_KC, false>), grid, dim3(256), 0, st, g);
    else hipLaunchKernelGGL((gemm_kernel_dma<T, A_KC, B_KC, true>), grid, dim3(256), 0, st, g);
    CHN_TRY(check_launch("gemm (direct-to-LDS)"));
    if (g.splits > 1) {
      const int64_t n = (int64_t)g.M * (g.ldp / 4);
      hipLaunchKernelGGL(gemm_splitk_finish_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, g);
      return check_launch("gemm split-K finish");
    }
    return CHN_OK;
  } else {
    return fail(CHN_ERR_LAUNCH, "gemm: internal: no direct-to-LDS kernel for this layout");
  }
}

template <typename T, int TM, int TN, bool A_KC, bool B_KC, int PB, int PB2 = PB>
chn_status launch_piece(const GemmArgs &g, hipStream_t st) {
  constexpr int LDS = 2 * (64 * TM + 64 * TN) * 128;
  static_assert(4 * kEpiStageBytes<TM, TN> <= LDS, "epilogue staging must fit in the operand stages");
  auto kern = gemm_kernel<T, TM, TN, A_KC, B_KC, PB, PB2>;
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
  if constexpr (TM == 1) {
    // one operand that only allows element-wise loads (a K of 10, say) does not slow down the other's
    if (g.piece_a == (int)sizeof(T) && g.piece_b == 16) return launch_piece<T, 1, 1, A_KC, B_KC, (int)sizeof(T), 16>(g, st);
    if (g.piece_a == 16 && g.piece_b == (int)sizeof(T)) return launch_piece<T, 1, 1, A_KC, B_KC, 16, (int)sizeof(T)>(g, st);
  }
  if (g.piece == 16) return launch_piece<T, TM, TN, A_KC, B_KC, 16>(g, st);
  if (g.piece == 8) return launch_piece<T, TM, TN, A_KC, B_KC, 8>(g, st);
  if constexpr (TM == 1) return launch_piece<T, 1, 1, A_KC, B_KC, (int)sizeof(T)>(g, st);
  else return fail(CHN_ERR_LAUNCH, "gemm: internal: element-wise loads only exist for the 64x64 tile");
}

template <typename T, bool A_KC, bool B_KC>
chn_status launch_layout(GemmArgs &g, hipStream_t st) {
  if ((int64_t)g.tiles_m * g.tiles_n * g.splits > 0x7fffffff) return fail(CHN_ERR_SHAPE, "gemm: too many tiles");
  if constexpr (sizeof(T) == 2) {
    if ((g.tile == 2 || g.tile == 3) && g.piece == 16 && g.dma && g.w8) return launch_w8<A_KC, B_KC>(g, st);
    if (g.tile == 3) return fail(CHN_ERR_LAUNCH, "gemm: the 256 x 128 tile needs the eight-wave direct-copy kernel");
  }
  if constexpr (kHasDmaKernel<T, A_KC, B_KC>) {
    if (g.tile == 2 && g.piece == 16 && g.dma) return launch_dma<T, A_KC, B_KC>(g, st);
  }
  if (g.tile == 2) return launch_tile<T, 4, 4, A_KC, B_KC>(g, st);
  if (g.tile == 1) return launch_tile<T, 2, 2, A_KC, B_KC>(g, st);
  return launch_tile<T, 1, 1, A_KC, B_KC>(g, st);
}

}  // namespace gemm
}  // namespace chn
