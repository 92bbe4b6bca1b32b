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
#include "common.h"

namespace chn {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct GemmArgs {
  const void *A, *B;
  void *C;
  int M, N, K;
  int64_t lda, ldb, ldc;  // elements; for a K-contiguous operand the stride between rows (m or n),
                          // otherwise the stride between consecutive k
  float alpha, beta;
  int epi;
  int c_bf16;             // C / aux / preact dtype: 0 fp32, 1 bf16
  const float *bias;
  const void *aux;
  int64_t ldaux;
  void *pre;
  int64_t ldpre;
  int avec, bvec;         // widest aligned global load per operand: 0 element, 1 8-byte, 2 16-byte
  int tiles_m, tiles_n;
};

template <typename T> struct Traits;
template <> struct Traits<float> { static constexpr int EPC = 4; };      // elements per 16-byte chunk
template <> struct Traits<bf16_raw> { static constexpr int EPC = 8; };

__device__ __forceinline__ int lds_off(int row, int q) { return row * 128 + ((q ^ ((row >> 1) & 7)) << 4); }

// Load EPC consecutive elements starting at p (all in range), using the widest access `vec` allows.
template <typename T>
__device__ __forceinline__ uint4 load_chunk(const T *p, int vec) {
  uint4 r;
  if (vec == 2) {
    r = *reinterpret_cast<const uint4 *>(p);
  } else if (vec == 1) {
    const uint2 lo = *reinterpret_cast<const uint2 *>(p);
    const uint2 hi = *reinterpret_cast<const uint2 *>(reinterpret_cast<const char *>(p) + 8);
    r = make_uint4(lo.x, lo.y, hi.x, hi.y);
  } else if constexpr (sizeof(T) == 4) {
    const uint32_t *q = reinterpret_cast<const uint32_t *>(p);
    r = make_uint4(q[0], q[1], q[2], q[3]);
  } else {
    const uint16_t *q = reinterpret_cast<const uint16_t *>(p);
    r = make_uint4(q[0] | ((uint32_t)q[1] << 16), q[2] | ((uint32_t)q[3] << 16),
                   q[4] | ((uint32_t)q[5] << 16), q[6] | ((uint32_t)q[7] << 16));
  }
  return r;
}

// Same, but elements at index >= limit (counted from p) read as zero.
template <typename T>
__device__ __forceinline__ uint4 load_chunk_guarded(const T *p, int limit) {
  constexpr int EPC = Traits<T>::EPC;
  uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
  for (int e = 0; e < EPC; ++e) {
    if (e < limit) {
      if constexpr (sizeof(T) == 4) w[e] = reinterpret_cast<const uint32_t *>(p)[e];
      else w[e >> 1] |= (uint32_t) reinterpret_cast<const uint16_t *>(p)[e] << ((e & 1) * 16);
    }
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

// One operand tile: ROWS rows (m or n) x 128 bytes of k.  NS 16-byte registers per thread.
template <typename T, int ROWS, bool KC>
struct TileLoader {
  static constexpr int EPC = Traits<T>::EPC;
  static constexpr int NS = ROWS / 32;                      // ROWS * 8 chunks / 256 threads
  static constexpr int NBLK = 8 * ROWS / EPC;               // EPC x EPC transpose blocks per tile
  static constexpr int NB = (NBLK + 255) / 256;             // ... per thread
  uint4 reg[KC ? NS : NB * EPC];

  // rows_total: extent of the operand along m (or n); row0: first row of this tile; k0: first k.
  __device__ __forceinline__ void load(const T *base, int64_t ld, int rows_total, int row0, int K, int k0, int vec) {
    if constexpr (KC) {
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        const int s = threadIdx.x + i * 256;
        const int row = row0 + (s >> 3), k = k0 + (s & 7) * EPC;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (row < rows_total && k < K) {
          const T *p = base + (int64_t)row * ld + k;
          v = (k + EPC <= K) ? load_chunk<T>(p, vec) : load_chunk_guarded<T>(p, K - k);
        }
        reg[i] = v;
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
          uint4 v = make_uint4(0, 0, 0, 0);
          if (blk < NBLK && k < K && m < rows_total) {
            const T *p = base + (int64_t)k * ld + m;
            v = (m + EPC <= rows_total) ? load_chunk<T>(p, vec) : load_chunk_guarded<T>(p, rows_total - m);
          }
          reg[b * EPC + j] = v;
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

template <typename T, int TM, int TN, bool A_KC, bool B_KC>
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
  TileLoader<T, BM, A_KC> la;
  TileLoader<T, BN, B_KC> lb;

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
  la.load(A, g.lda, g.M, m0, g.K, 0, g.avec);
  lb.load(B, g.ldb, g.N, n0, g.K, 0, g.bvec);
  la.store(lds);
  lb.store(lds + A_BYTES);
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    char *cur = lds + (kt & 1) * STAGE;
    char *nxt = lds + ((kt + 1) & 1) * STAGE;
    const bool more = kt + 1 < nk;
    if (more) {
      la.load(A, g.lda, g.M, m0, g.K, (kt + 1) * BK, g.avec);
      lb.load(B, g.ldb, g.N, n0, g.K, (kt + 1) * BK, g.bvec);
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

template <typename T, int TM, int TN, bool A_KC, bool B_KC>
chn_status launch_tile(const GemmArgs &g, hipStream_t st) {
  constexpr int LDS = 2 * (64 * TM + 64 * TN) * 128;
  auto kern = gemm_kernel<T, TM, TN, A_KC, B_KC>;
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

template <typename T, bool A_KC, bool B_KC>
chn_status launch_layout(GemmArgs &g, hipStream_t st) {
  auto tiles = [&](int b) { return (int64_t)((g.M + b - 1) / b) * ((g.N + b - 1) / b); };
  int64_t t;
  if ((t = tiles(256)) >= 192) {
    if (t > 0x7fffffff) return fail(CHN_ERR_SHAPE, "gemm: too many tiles");
    g.tiles_m = (g.M + 255) / 256; g.tiles_n = (g.N + 255) / 256;
    return launch_tile<T, 4, 4, A_KC, B_KC>(g, st);
  }
  if ((t = tiles(128)) >= 128) {
    g.tiles_m = (g.M + 127) / 128; g.tiles_n = (g.N + 127) / 128;
    return launch_tile<T, 2, 2, A_KC, B_KC>(g, st);
  }
  g.tiles_m = (g.M + 63) / 64; g.tiles_n = (g.N + 63) / 64;
  return launch_tile<T, 1, 1, A_KC, B_KC>(g, st);
}

template <typename T>
chn_status launch_dtype(GemmArgs &g, bool a_kc, bool b_kc, hipStream_t st) {
  if (a_kc && b_kc) return launch_layout<T, true, true>(g, st);
  if (a_kc && !b_kc) return launch_layout<T, true, false>(g, st);
  if (!a_kc && b_kc) return launch_layout<T, false, true>(g, st);
  return launch_layout<T, false, false>(g, st);
}

int vec_class(const void *p, int64_t ld_elems, int isz) {
  const uintptr_t a = reinterpret_cast<uintptr_t>(p);
  const int64_t ldb = ld_elems * isz;
  if (a % 16 == 0 && ldb % 16 == 0) return 2;
  if (a % 8 == 0 && ldb % 8 == 0) return 1;
  return 0;
}

}  // namespace
}  // namespace chn

extern "C" {

size_t chn_gemm_workspace_bytes(const chn_array *A, const chn_array *B, const chn_array *C) {
  (void)A; (void)B; (void)C;
  return 0;
}

chn_status chn_gemm(const chn_array *A, const chn_array *B, const chn_array *C, float alpha, float beta,
                    int epilogue, const chn_array *bias, const chn_array *aux, const chn_array *preact_out,
                    void *ws, size_t ws_bytes, chn_stream stream) {
  using namespace chn;
  (void)ws; (void)ws_bytes;
  CHN_TRY(validate(A, "A", false));
  CHN_TRY(validate(B, "B", false));
  CHN_TRY(validate(C, "C", true));
  if (A->ndim != 2 || B->ndim != 2 || C->ndim != 2) return fail(CHN_ERR_NDIM, "gemm: A, B and C must be 2-d");
  if (epilogue < 0 || epilogue >= CHN_EPI_COUNT_) return fail(CHN_ERR_OP, "gemm: unknown epilogue %d", epilogue);
  if (!is_float(A->dtype) || A->dtype != B->dtype) return fail(CHN_ERR_DTYPE, "gemm: A and B must share F32 or BF16");
  if (!is_float(C->dtype) || (A->dtype == CHN_F32 && C->dtype != CHN_F32))
    return fail(CHN_ERR_DTYPE, "gemm: C must be F32 (or BF16 when A and B are BF16)");
  const int64_t M = A->shape[0], K = A->shape[1], N = B->shape[1];
  if (B->shape[0] != K) return fail(CHN_ERR_SHAPE, "gemm: A is (%lld,%lld) but B has %lld rows", (long long)M, (long long)K, (long long)B->shape[0]);
  if (C->shape[0] != M || C->shape[1] != N) return fail(CHN_ERR_SHAPE, "gemm: C must be (%lld,%lld)", (long long)M, (long long)N);
  if (M > 0x3fffffff || N > 0x3fffffff || K > 0x3fffffff) return fail(CHN_ERR_SHAPE, "gemm: dimension too large");
  const int isz = dtype_size(A->dtype), csz = dtype_size(C->dtype);
  GemmArgs g{};
  int64_t cr, cc;
  CHN_TRY(row_major_2d(C, "C", &cr, &cc, &g.ldc));
  // operand layouts: which dimension has unit stride
  auto unit = [&](const chn_array *X, int d) { return X->shape[d] <= 1 || X->strides[d] == isz; };
  bool a_kc, b_kc;
  if (unit(A, 1)) { a_kc = true; g.lda = M > 1 ? A->strides[0] / isz : K; }
  else if (unit(A, 0)) { a_kc = false; g.lda = K > 1 ? A->strides[1] / isz : M; }
  else return fail(CHN_ERR_STRIDE, "gemm: A needs a unit-stride dimension");
  if (unit(B, 0)) { b_kc = true; g.ldb = N > 1 ? B->strides[1] / isz : K; }
  else if (unit(B, 1)) { b_kc = false; g.ldb = K > 1 ? B->strides[0] / isz : N; }
  else return fail(CHN_ERR_STRIDE, "gemm: B needs a unit-stride dimension");
  if ((a_kc && M > 1 && g.lda < K) || (!a_kc && K > 1 && g.lda < M) || (b_kc && N > 1 && g.ldb < K) || (!b_kc && K > 1 && g.ldb < N))
    return fail(CHN_ERR_STRIDE, "gemm: overlapping (broadcast) operand rows are not supported");
  const bool needs_bias = epilogue >= CHN_EPI_BIAS && epilogue <= CHN_EPI_BIAS_GELU;
  const bool needs_aux = epilogue == CHN_EPI_RELU_BWD || epilogue == CHN_EPI_GELU_BWD;
  if (needs_bias) {
    CHN_TRY(validate(bias, "bias", false));
    if (bias->dtype != CHN_F32) return fail(CHN_ERR_DTYPE, "gemm: bias must be F32");
    if (bias->ndim != 1 || bias->shape[0] != N || !is_contiguous(bias)) return fail(CHN_ERR_SHAPE, "gemm: bias must be a contiguous (%lld,) array", (long long)N);
    g.bias = static_cast<const float *>(bias->data);
  }
  if (needs_aux) {
    CHN_TRY(validate(aux, "aux", false));
    if (aux->dtype != C->dtype) return fail(CHN_ERR_DTYPE, "gemm: aux must have C's dtype");
    int64_t ar, ac;
    CHN_TRY(row_major_2d(aux, "aux", &ar, &ac, &g.ldaux));
    if (ar != M || ac != N) return fail(CHN_ERR_SHAPE, "gemm: aux must have C's shape");
    g.aux = aux->data;
  }
  if (preact_out) {
    if (epilogue != CHN_EPI_BIAS_GELU) return fail(CHN_ERR_OP, "gemm: preact_out is only produced by the BIAS_GELU epilogue");
    CHN_TRY(validate(preact_out, "preact_out", true));
    if (preact_out->dtype != C->dtype) return fail(CHN_ERR_DTYPE, "gemm: preact_out must have C's dtype");
    int64_t pr, pc;
    CHN_TRY(row_major_2d(preact_out, "preact_out", &pr, &pc, &g.ldpre));
    if (pr != M || pc != N) return fail(CHN_ERR_SHAPE, "gemm: preact_out must have C's shape");
    g.pre = preact_out->data;
  }
  if (M == 0 || N == 0) return CHN_OK;
  (void)csz;
  g.A = A->data; g.B = B->data; g.C = C->data;
  g.M = (int)M; g.N = (int)N; g.K = (int)K;
  g.alpha = alpha; g.beta = beta; g.epi = epilogue; g.c_bf16 = C->dtype == CHN_BF16;
  g.avec = vec_class(A->data, g.lda, isz);
  g.bvec = vec_class(B->data, g.ldb, isz);
  hipStream_t st = as_stream(stream);
  if (A->dtype == CHN_F32) return launch_dtype<float>(g, a_kc, b_kc, st);
  return launch_dtype<bf16_raw>(g, a_kc, b_kc, st);
}

}  // extern "C"
