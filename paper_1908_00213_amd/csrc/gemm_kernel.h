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
//   * the K loop advances 128 bytes of K per operand row per step (64 bf16 or 32 fp32).  Operand
//     tiles live in LDS as rows of 128 bytes = 8 chunks of 16 bytes, always K-packed, with the chunk
//     index XOR-swizzled by (row/2)%8 so that neither the 16-byte stores nor the 16-byte MFMA
//     fragment reads collide on LDS banks, without padding;
//   * operands whose unit stride runs along K are copied chunk by chunk; operands whose unit stride
//     runs along M/N (transposed views) are loaded in 16-byte pieces along M/N and transposed in
//     registers (8x8 bf16 or 4x4 fp32 blocks) on their way into LDS, so the inner loop is the same
//     for all four layout combinations and no second copy of an operand is ever made;
//   * global loads for step t+1 are issued into registers before the MFMAs of step t and written to
//     the other LDS buffer after them: one barrier per step;
//   * since the sum over k is order-free, the 16 (8) k-values one lane feeds to an MFMA need not be
//     the hardware's nominal ones as long as A and B agree; each lane therefore reads one whole
//     16-byte chunk per 32 rows and step;
//   * workgroups are renumbered so that the eight XCDs (which take consecutive workgroup ids
//     round-robin) each work on a compact patch of C tiles and share operand tiles in their own L2.
// The epilogue applies alpha/beta, bias, activation or activation-gradient in fp32 and rounds once.
#pragma once
#include "common.h"
#include "gemm_args.h"

namespace chn {
namespace gemm {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));


template <typename T> struct Traits;
template <> struct Traits<float> { static constexpr int EPC = 4; };      // elements per 16-byte chunk
template <> struct Traits<bf16_raw> { static constexpr int EPC = 8; };

__device__ __forceinline__ int lds_off(int row, int q) { return row * 128 + ((q ^ ((row >> 1) & 7)) << 4); }

// Sixteen zero bytes in device memory: out-of-range pieces are redirected here, so that the loaded
// value needs no masking (a select on loaded data would force the wave to wait for the load at once).
__device__ const uint4 kZeroChunk = {0u, 0u, 0u, 0u};

// Load one 16-byte chunk (EPC consecutive elements starting at p) in pieces of PB bytes without any
// branch: a piece whose first element index is >= n_valid is read from the zero chunk instead.
// Pieces never straddle the valid range because the host only picks a piece size that divides the
// operand's extent along its unit-stride dimension.
// Loads go through pointers that carry the global address space explicitly: a generic ("flat") load
// would also count against the LDS counter and make every wait for an LDS read wait for HBM as well.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <typename V>
__device__ __forceinline__ V global_load(uintptr_t addr) {
  return *reinterpret_cast<const __attribute__((address_space(1))) V *>(addr);
}

template <typename T, int PB>
__device__ __forceinline__ uint4 load_chunk(const T *p, int n_valid) {
  constexpr int PE = PB / (int)sizeof(T);   // elements per piece
  constexpr int NP = 16 / PB;               // pieces per chunk
  const uintptr_t zero = reinterpret_cast<uintptr_t>(&kZeroChunk);
  uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int j = 0; j < NP; ++j) {
    const uintptr_t q = (j * PE < n_valid) ? reinterpret_cast<uintptr_t>(p + j * PE) : zero;
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
// and LDS.
template <typename T, int ROWS, bool KC, int PB>
struct TileLoader {
  static constexpr int EPC = Traits<T>::EPC;
  static constexpr int NS = ROWS / 32;                      // ROWS * 8 chunks / 256 threads
  static constexpr int NBLK = 8 * ROWS / EPC;               // EPC x EPC transpose blocks per tile
  static constexpr int NB = (NBLK + 255) / 256;             // ... per thread
  uint4 reg[KC ? NS : NB * EPC];

  // rows_total: extent of the operand along m (or n); row0: first row of this tile; k0: first k.
  __device__ __forceinline__ void load(const T *base, int64_t ld, int rows_total, int row0, int K, int k0) {
    if constexpr (KC) {
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        const int s = threadIdx.x + i * 256;
        const int row = row0 + (s >> 3), k = k0 + (s & 7) * EPC;
        const int n_valid = row < rows_total ? K - k : 0;
        reg[i] = load_chunk<T, PB>(base + (int64_t)row * ld + k, n_valid);
      }
    } else {
      // blocks of EPC (k) x EPC (m): EPC loads of 16 bytes along m, one per k
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const int blk = threadIdx.x + b * 256;
        const int kg = blk & 7, mc = blk >> 3;
        const int m = row0 + mc * EPC;
#pragma unroll
        for (int j = 0; j < EPC; ++j) {
          const int k = k0 + kg * EPC + j;
          const int n_valid = (blk < NBLK && k < K) ? rows_total - m : 0;
          reg[b * EPC + j] = load_chunk<T, PB>(base + (int64_t)k * ld + m, n_valid);
        }
      }
    }
  }

  __device__ __forceinline__ void store(char *lds) const {
    if constexpr (KC) {
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        const int s = threadIdx.x + i * 256;
        *reinterpret_cast<uint4 *>(lds + lds_off(s >> 3, s & 7)) = reg[i];
      }
    } else {
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const int blk = threadIdx.x + b * 256;
        if (blk >= NBLK) continue;
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
              const uint32_t lo = (&r[2 * q].x)[e >> 1], hi = (&r[2 * q + 1].x)[e >> 1];
              w[q] = (e & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
            }
            o = make_uint4(w[0], w[1], w[2], w[3]);
          }
          *reinterpret_cast<uint4 *>(lds + lds_off(mc * EPC + e, kg)) = o;
        }
      }
    }
  }
};

__device__ __forceinline__ float act_load(const void *p, int64_t idx, int is_bf16) {
  return is_bf16 ? bf16_to_f32(static_cast<const bf16_raw *>(p)[idx]) : static_cast<const float *>(p)[idx];
}

__device__ __forceinline__ void out_store(void *p, int64_t idx, int is_bf16, float v) {
  if (is_bf16) static_cast<bf16_raw *>(p)[idx] = f32_to_bf16(v);
  else static_cast<float *>(p)[idx] = v;
}

// Epilogue of one 32x32 accumulator block: this lane's 16 values sit in column `col`, rows
// row_base + 8*(v/4) + v%4.
__device__ __forceinline__ void epilogue_block(const GemmArgs &g, const floatx16 &a, int row_base, int col) {
  if (col >= g.N) return;
  const float bias = (g.epi >= CHN_EPI_BIAS && g.epi <= CHN_EPI_BIAS_GELU) ? g.bias[col] : 0.0f;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int row = row_base + 8 * (v >> 2) + (v & 3);
    if (row < g.M) {
      const int64_t ci = (int64_t)row * g.ldc + col;
      float x = g.alpha * a[v];
      if (g.beta != 0.0f) x += g.beta * act_load(g.C, ci, g.c_bf16);
      x += bias;
      if (g.epi == CHN_EPI_BIAS_RELU) {
        x = fmaxf(x, 0.0f);
      } else if (g.epi == CHN_EPI_BIAS_GELU) {
        if (g.pre) out_store(g.pre, (int64_t)row * g.ldpre + col, g.c_bf16, x);
        x = gelu_f(x);
      } else if (g.epi == CHN_EPI_RELU_BWD) {
        x = act_load(g.aux, (int64_t)row * g.ldaux + col, g.c_bf16) > 0.0f ? x : 0.0f;
      } else if (g.epi == CHN_EPI_GELU_BWD) {
        x *= gelu_grad_f(act_load(g.aux, (int64_t)row * g.ldaux + col, g.c_bf16));
      }
      out_store(g.C, ci, g.c_bf16, x);
    }
  }
}

template <typename T, int TM, int TN, bool A_KC, bool B_KC, int PB>
__global__ __launch_bounds__(256) void gemm_kernel(GemmArgs g) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  constexpr int BK = 128 / sizeof(T);               // elements of k per step
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
  extern __shared__ __align__(16) char lds[];

  // ---- which C tile: XCD-aware renumbering, then grouped (8 tile rows at a time) ordering
  const int nb = g.tiles_m * g.tiles_n;
  int pid = blockIdx.x;
  const int nb8 = nb & ~7;
  if (pid < nb8) pid = (pid & 7) * (nb8 >> 3) + (pid >> 3);
  constexpr int GROUP = 8;
  const int width = GROUP * g.tiles_n;
  const int first_m = (pid / width) * GROUP;
  const int gsize = min(g.tiles_m - first_m, GROUP);
  const int tm = first_m + (pid % width) % gsize;
  const int tn = (pid % width) / gsize;
  const int m0 = tm * BM, n0 = tn * BN;

  const T *A = static_cast<const T *>(g.A);
  const T *B = static_cast<const T *>(g.B);
  TileLoader<T, BM, A_KC, PB> la;
  TileLoader<T, BN, B_KC, PB> lb;

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

  const int nk = (g.K + BK - 1) / BK;
  la.load(A, g.lda, g.M, m0, g.K, 0);
  lb.load(B, g.ldb, g.N, n0, g.K, 0);
  la.store(lds);
  lb.store(lds + A_BYTES);
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    char *cur = lds + (kt & 1) * STAGE;
    char *nxt = lds + ((kt + 1) & 1) * STAGE;
    const bool more = kt + 1 < nk;
    if (more) {
      la.load(A, g.lda, g.M, m0, g.K, (kt + 1) * BK);
      lb.load(B, g.ldb, g.N, n0, g.K, (kt + 1) * BK);
    }
    const char *sa = cur + (wm * TM * 32 + r) * 128;
    const char *sb = cur + A_BYTES + (wn * TN * 32 + r) * 128;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      uint4 fa[TM], fb[TN];
      const int q = ks * 2 + h;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = wm * TM * 32 + i * 32 + r;
        fa[i] = *reinterpret_cast<const uint4 *>(sa + i * 32 * 128 + ((q ^ ((row >> 1) & 7)) << 4));
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int row = wn * TN * 32 + j * 32 + r;
        fb[j] = *reinterpret_cast<const uint4 *>(sb + j * 32 * 128 + ((q ^ ((row >> 1) & 7)) << 4));
      }
      if constexpr (sizeof(T) == 2) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[i]),
                                                                __builtin_bit_cast(bf16x8, fb[j]), acc[i][j], 0, 0, 0);
      } else {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float((&fa[i].x)[kk]),
                                                               __uint_as_float((&fb[j].x)[kk]), acc[i][j], 0, 0, 0);
      }
    }
    if (more) {
      la.store(nxt);
      lb.store(nxt + A_BYTES);
    }
    __syncthreads();
  }

  // ---- epilogue: lane holds, per 32x32 block, column r and rows 8*(v/4) + 4*h + v%4
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
      epilogue_block(g, acc[i][j], m0 + wm * TM * 32 + i * 32 + 4 * h, n0 + wn * TN * 32 + j * 32 + r);
}

template <typename T, int TM, int TN, bool A_KC, bool B_KC, int PB>
chn_status launch_piece(const GemmArgs &g, hipStream_t st) {
  constexpr int LDS = 2 * (64 * TM + 64 * TN) * 128;
  auto kern = gemm_kernel<T, TM, TN, A_KC, B_KC, PB>;
  static bool configured = false;  // per instantiation
  if (!configured) {
    if (LDS > 64 * 1024) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
      if (e != hipSuccess) return fail(CHN_ERR_LAUNCH, "gemm: cannot reserve %d bytes of LDS: %s", LDS, hipGetErrorString(e));
    }
    configured = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)(g.tiles_m * g.tiles_n)), dim3(256), LDS, st, g);
  return check_launch("gemm");
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
  auto tiles = [&](int b) { return (int64_t)((g.M + b - 1) / b) * ((g.N + b - 1) / b); };
  int64_t t;
  const bool wide = g.piece >= 8;   // operands that need element-wise loads only get the small tile
  if (wide && (t = tiles(256)) >= 192) {
    if (t > 0x7fffffff) return fail(CHN_ERR_SHAPE, "gemm: too many tiles");
    g.tiles_m = (g.M + 255) / 256; g.tiles_n = (g.N + 255) / 256;
    return launch_tile<T, 4, 4, A_KC, B_KC>(g, st);
  }
  if (wide && (t = tiles(128)) >= 128) {
    g.tiles_m = (g.M + 127) / 128; g.tiles_n = (g.N + 127) / 128;
    return launch_tile<T, 2, 2, A_KC, B_KC>(g, st);
  }
  g.tiles_m = (g.M + 63) / 64; g.tiles_n = (g.N + 63) / 64;
  return launch_tile<T, 1, 1, A_KC, B_KC>(g, st);
}

}  // namespace gemm
}  // namespace chn
