// chn_gemm: host side of the dense product -- validation, layout classification and dispatch to the
// kernel families in gemm_kernel.h (one object file per dtype and operand layout).
#include <atomic>

#include "common.h"
#include "gemm_args.h"

namespace chn {
namespace gemm {

#define CHN_DECL(name) chn_status name(GemmArgs &g, hipStream_t st);
CHN_DECL(launch_f32_kk) CHN_DECL(launch_f32_km) CHN_DECL(launch_f32_mk) CHN_DECL(launch_f32_mm)
CHN_DECL(launch_bf16_kk) CHN_DECL(launch_bf16_km) CHN_DECL(launch_bf16_mk) CHN_DECL(launch_bf16_mm)
#undef CHN_DECL

}  // namespace gemm
}  // namespace chn

namespace chn {
namespace {

using gemm::GemmArgs;

// chn_gemm_plan_override: what tests force instead of the planner's choice (-1: not forced)
std::atomic<int> g_force_tile{-1}, g_force_splits{-1}, g_force_direct{-1};
constexpr double kNarrowStep = 0.92, kNarrowFixed = 12.0;   // microseconds per tile step / per block of the 256 x 128 tile
std::atomic<int> g_force_w8{-1};

// Largest load piece (bytes) that is aligned for every row start of the operand and divides its
// extent along the unit-stride dimension, so that a piece is never partly out of range.
// overhang: the extent need not be a multiple of the piece.  The last piece of a row then also brings
// what follows the row in memory (the padding of a pitched row, or the next row's first elements;
// never another page: the piece is aligned to its own size).  That is harmless exactly where the
// unit stride runs along M or N: those values become rows of A (columns of B) beyond M (N), and
// the rows (columns) of C they feed are never stored.
int piece_bytes(const void *p, int64_t ld_elems, int64_t extent_elems, int isz, bool overhang) {
  const uintptr_t a = reinterpret_cast<uintptr_t>(p);
  const int64_t ldb = ld_elems * isz, ext = extent_elems * isz;
  if (a % 16 == 0 && ldb % 16 == 0 && (overhang || ext % 16 == 0)) return 16;
  if (a % 8 == 0 && ldb % 8 == 0 && (overhang || ext % 8 == 0)) return 8;
  return isz;
}

// Operand layouts (which dimension has unit stride), leading dimensions and load piece size.
chn_status classify(const chn_array *A, const chn_array *B, GemmArgs *g, bool *a_kc, bool *b_kc) {
  const int isz = dtype_size(A->dtype);
  const int64_t M = A->shape[0], K = A->shape[1], N = B->shape[1];
  auto unit = [&](const chn_array *X, int d) { return X->shape[d] <= 1 || X->strides[d] == isz; };
  if (unit(A, 1)) { *a_kc = true; g->lda = M > 1 ? A->strides[0] / isz : K; }
  else if (unit(A, 0)) { *a_kc = false; g->lda = K > 1 ? A->strides[1] / isz : M; }
  else return fail(CHN_ERR_STRIDE, "gemm: A needs a unit-stride dimension");
  if (unit(B, 0)) { *b_kc = true; g->ldb = N > 1 ? B->strides[1] / isz : K; }
  else if (unit(B, 1)) { *b_kc = false; g->ldb = K > 1 ? B->strides[0] / isz : N; }
  else return fail(CHN_ERR_STRIDE, "gemm: B needs a unit-stride dimension");
  if ((*a_kc && M > 1 && g->lda < K) || (!*a_kc && K > 1 && g->lda < M) || (*b_kc && N > 1 && g->ldb < K) || (!*b_kc && K > 1 && g->ldb < N))
    return fail(CHN_ERR_STRIDE, "gemm: overlapping (broadcast) operand rows are not supported");
  const int pa = piece_bytes(A->data, g->lda, *a_kc ? K : M, isz, false);
  const int pb = piece_bytes(B->data, g->ldb, *b_kc ? K : N, isz, false);
  g->piece_exact = pa < pb ? pa : pb;
  // the kernels that stage operands in registers take pieces that hang over the end of a row of an
  // operand whose unit stride runs along M or N
  const int qa = piece_bytes(A->data, g->lda, *a_kc ? K : M, isz, !*a_kc);
  const int qb = piece_bytes(B->data, g->ldb, *b_kc ? K : N, isz, !*b_kc);
  g->piece = qa < qb ? qa : qb;
  g->piece_a = qa; g->piece_b = qb;
  if (K == 0) { *a_kc = *b_kc = true; g->piece = g->piece_exact = g->piece_a = g->piece_b = isz; }  // nothing to multiply: every load is redirected to zeros
  g->M = (int)M; g->N = (int)N; g->K = (int)K;
  return CHN_OK;
}

// Whether the direct-copy 256x256 kernel can take the product: it needs 16-byte pieces (so K is a
// multiple of the chunk length for K-contiguous operands) and 32-bit offsets inside a tile; fp32 needs
// at least one K-contiguous operand for it.
bool direct_copy_fits(const GemmArgs &g, int isz, bool a_kc, bool b_kc) {
  const bool dma_on = g_force_direct.load(std::memory_order_relaxed) != 0;
  const int64_t max_ld = (int64_t)0xffffffffu / (256 * isz);
  return dma_on && g.piece_exact == 16 && g.K > 0 && g.lda < max_ld && g.ldb < max_ld && (isz == 2 || a_kc || b_kc);
}

// Macro tile (3: 256x128, 2: 256x256, 1: 128x128, 0: 64x64) and number of K splits, chosen by a small cost model
// from measured figures: every compute unit works through its share of the blocks one after another,
// a block costing a fixed part (launch, prologue, epilogue) plus its tile steps times the time one
// compute unit needs per tile step of that tile and kernel (for the smaller tiles, of which several
// run on a compute unit at once, the amortised figure).  A problem with too few tiles to occupy 256
// compute units but a long K is cut along K: every split writes fp32 partial sums to the workspace and
// a second kernel adds them in a fixed order and runs the epilogue (its traffic and launch are charged
// to the split candidates).
void plan(GemmArgs *g, int isz, bool a_kc, bool b_kc, bool allow_split, bool big_unsplit = false) {
  // microseconds per tile step [tile][0: both operands K-contiguous, 1: one, 2: none] and per block
  static const double step_bf16[3][3] = {{0.27, 0.33, 0.56}, {0.57, 0.68, 1.12}, {1.90, 2.25, 2.70}};
  static const double step_f32[3][3] = {{0.52, 0.62, 0.65}, {1.95, 2.40, 2.10}, {6.90, 7.50, 7.90}};
  static const double fixed_bf16[3] = {1.0, 3.0, 12.0}, fixed_f32[3] = {1.5, 4.0, 18.0};
  const double step_direct = 1.48;                        // bf16 direct-copy kernel, any layout
  const int lay = (a_kc ? 0 : 1) + (b_kc ? 0 : 1);
  const bool direct = direct_copy_fits(*g, isz, a_kc, b_kc);
  const bool wide = g->piece >= 8;   // operands that need element-wise loads only get the small tile
  const double narrow = g->piece >= 16 ? 1.0 : g->piece >= 8 ? 1.15 : 2.0;   // more, smaller loads per step
  const int nk = (g->K + 128 / isz - 1) / (128 / isz);   // tile steps along K
  static const int split_choices[] = {1, 2, 3, 4, 5, 6, 7, 8, 10, 12, 14, 16};
  double best = 1e300;
  g->tile = 0; g->splits = 1;
  for (int tile = wide ? 2 : 0; tile >= 0; --tile) {
    const int b = 64 << tile;
    const int64_t tiles = (int64_t)((g->M + b - 1) / b) * ((g->N + b - 1) / b);
    double per_step = (isz == 2 ? step_bf16 : step_f32)[tile][lay] * narrow;
    if (tile == 2 && direct && isz == 2) per_step = step_direct;
    const double fixed = (isz == 2 ? fixed_bf16 : fixed_f32)[tile];
    for (int s : split_choices) {
      if (s > 1 && (!allow_split || s > nk / 4)) break;
      const int64_t blocks = tiles * s;
      const int steps = (nk + s - 1) / s;
      // Up to `conc` blocks of this tile run on a compute unit at once, each then `conc` times slower
      // per step than the amortised figure; a lone block only `slow` times (it is not that much faster
      // alone), in between linearly.  Full rounds of 256 * conc blocks, then the remainder.
      const int conc = tile == 2 ? 1 : tile == 1 ? 2 : 4;
      const double slow = tile == 2 ? 1.0 : tile == 1 ? 1.5 : 1.6;   // (64x64: 2.0 before the kernel looked two tiles ahead)
      const int64_t full = blocks / (256 * conc), rem = blocks % (256 * conc);
      double t = (double)full * (fixed + steps * per_step * conc);
      if (rem > 0) {
        const int per_cu = (int)((rem + 255) / 256);
        const double f = conc == 1 ? 1.0 : slow + (conc - slow) * (per_cu - 1) / (conc - 1);
        t += fixed + steps * per_step * f;
      }
      t *= 1e-6;
      if (s > 1) t += 10e-6 + (double)(s + 1) * g->M * g->N * 4.0 / 4e12;
      if (t < best * 0.97) { best = t; g->tile = tile; g->splits = s; }   // prefer larger tiles / fewer splits on near-ties
    }
  }
  // The 256 x 128 tile of the eight-wave kernel (bf16, both operands K-contiguous): taken when it fills the chip
  // in one round without a cut along K where the square tile cannot (N near 1000 with a long M).
  const bool narrow_ok = direct && isz == 2 && a_kc && b_kc && !big_unsplit && g_force_w8.load(std::memory_order_relaxed) != 0;
  if (narrow_ok) {
    const int64_t tiles = (int64_t)((g->M + 255) / 256) * ((g->N + 127) / 128);
    const int64_t rounds = (tiles + 255) / 256;
    const double t = (double)rounds * (kNarrowFixed + nk * kNarrowStep) * 1e-6;
    if (t < best * 0.97) { best = t; g->tile = 3; g->splits = 1; }
  }
  {   // chn_gemm_plan_override
    const int force_tile = g_force_tile.load(std::memory_order_relaxed), force_splits = g_force_splits.load(std::memory_order_relaxed);
    if (force_tile >= 0 && force_tile <= (wide ? 2 : 0)) g->tile = force_tile;
    if (force_tile == 3 && narrow_ok) g->tile = 3;
    if (force_tile >= 0 && force_tile != 3 && g->tile == 3) g->tile = wide ? 2 : 0;
    if (force_splits >= 1 && allow_split && force_splits <= nk) g->splits = force_splits;
  }
  if (big_unsplit) { g->tile = 2; g->splits = 1; }        // (the caller has checked that the operands allow the big tile)
  const int bm = g->tile == 3 ? 256 : 64 << g->tile, bn = g->tile == 3 ? 128 : 64 << g->tile;
  g->tiles_m = (g->M + bm - 1) / bm;
  g->tiles_n = (g->N + bn - 1) / bn;
  g->ldp = (g->N + 3) & ~3;
  g->dma = (g->tile == 2 || g->tile == 3) && direct;
}

// Which of the two direct-copy kernels takes a bf16 product on the 256x256 tile: the eight-wave one.  Both
// are bound by the chip's power limit on random data and within 2 % of each other on the long products of
// the wide-MLP step (three machines: the eight-wave kernel ahead by 1-2 % on two, behind by 1.5 % on one);
// where a workgroup's fixed parts weigh more the eight-wave kernel wins clearly -- its two waves per SIMD
// overlap prologue, epilogue and barriers: 8192x4096x1000 in 95-100 us against 118-120 us, the products
// with an activation-gradient epilogue 3-5 % faster.  The four-wave kernel (a third less LDS traffic per
// MFMA) stays for fp32 and as the forced alternative of the tests.
bool eight_waves(const GemmArgs &g, int isz, int epilogue) {
  if (!g.dma || isz != 2) return false;
  const int f = g_force_w8.load(std::memory_order_relaxed);
  (void)epilogue;
  return f < 0 || f != 0;
}

size_t split_bytes(const GemmArgs &g) {
  return g.splits > 1 ? (size_t)g.splits * g.M * g.ldp * sizeof(float) : 0;
}

}  // namespace
}  // namespace chn

extern "C" {

size_t chn_gemm_workspace_bytes(const chn_array *A, const chn_array *B, const chn_array *C) {
  using namespace chn;
  if (!A || !B || !C || A->ndim != 2 || B->ndim != 2 || !is_float(A->dtype) || A->dtype != B->dtype) return 0;
  if (A->shape[1] != B->shape[0] || A->shape[0] <= 0 || B->shape[1] <= 0) return 0;
  if (A->shape[0] > 0x3fffffff || A->shape[1] > 0x3fffffff || B->shape[1] > 0x3fffffff) return 0;
  GemmArgs g{};
  bool a_kc, b_kc;
  if (classify(A, B, &g, &a_kc, &b_kc) != CHN_OK) return 0;
  plan(&g, dtype_size(A->dtype), a_kc, b_kc, true);
  return split_bytes(g);
}

void chn_gemm_plan_override(int tile, int splits, int direct_copy) {
  chn::g_force_tile.store(tile, std::memory_order_relaxed);
  chn::g_force_splits.store(splits, std::memory_order_relaxed);
  chn::g_force_direct.store(direct_copy >= 2 ? 1 : direct_copy, std::memory_order_relaxed);
  chn::g_force_w8.store(direct_copy == 2 ? 0 : direct_copy == 3 ? 1 : -1, std::memory_order_relaxed);
}

int chn_gemm_plan(const chn_array *A, const chn_array *B, const chn_array *C, int have_workspace) {
  using namespace chn;
  CHN_TRY(validate(A, "A", false));
  CHN_TRY(validate(B, "B", false));
  CHN_TRY(validate(C, "C", true));
  if (A->ndim != 2 || B->ndim != 2 || C->ndim != 2) return fail(CHN_ERR_NDIM, "gemm: A, B and C must be 2-d");
  if (!is_float(A->dtype) || A->dtype != B->dtype) return fail(CHN_ERR_DTYPE, "gemm: A and B must share F32 or BF16");
  if (A->shape[1] != B->shape[0] || C->shape[0] != A->shape[0] || C->shape[1] != B->shape[1]) return fail(CHN_ERR_SHAPE, "gemm: shapes do not match");
  if (A->shape[0] > 0x3fffffff || A->shape[1] > 0x3fffffff || B->shape[1] > 0x3fffffff) return fail(CHN_ERR_SHAPE, "gemm: dimension too large");
  GemmArgs g{};
  bool a_kc, b_kc;
  CHN_TRY(classify(A, B, &g, &a_kc, &b_kc));
  const int isz = dtype_size(A->dtype);
  plan(&g, isz, a_kc, b_kc, have_workspace != 0);
  return g.tile | (g.dma ? 4 : 0) | (eight_waves(g, isz, CHN_EPI_NONE) ? 8 : 0) | (g.splits << 4);
}

chn_status chn_gemm(const chn_array *A, const chn_array *B, const chn_array *C, float alpha, float beta,
                    int epilogue, const chn_array *bias, const chn_array *aux, const chn_array *preact_out,
                    void *ws, size_t ws_bytes, chn_stream stream) {
  using namespace chn;
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
  bool a_kc, b_kc;
  CHN_TRY(classify(A, B, &g, &a_kc, &b_kc));
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
  if (epilogue == CHN_EPI_BF16_COPY && !preact_out) return fail(CHN_ERR_NULL, "gemm: the BF16_COPY epilogue needs preact_out");
  bool want_colsum = false;
  if (preact_out && needs_aux) {
    // activation-gradient epilogues: the second output holds column sums of C over blocks of 128 rows
    CHN_TRY(validate(preact_out, "preact_out", true));
    if (preact_out->dtype != CHN_F32) return fail(CHN_ERR_DTYPE, "gemm: the row-block column sums must be F32");
    int64_t pr, pc;
    CHN_TRY(row_major_2d(preact_out, "preact_out", &pr, &pc, &g.ldcs));
    if (M % 256 || N % 256 || pr != M / 128 || pc != N)
      return fail(CHN_ERR_SHAPE, "gemm: row-block column sums need M and N to be multiples of 256 and an (M/128, N) array");
    if (beta != 0.0f) return fail(CHN_ERR_OP, "gemm: row-block column sums are not produced together with beta != 0");
    if (reinterpret_cast<uintptr_t>(preact_out->data) % 16 || g.ldcs % 4)
      return fail(CHN_ERR_STRIDE, "gemm: the row-block column sums need 16-byte aligned rows");
    g.colsum = static_cast<float *>(preact_out->data);
    want_colsum = true;
  } else if (preact_out) {
    if (epilogue != CHN_EPI_BIAS_GELU && epilogue != CHN_EPI_BF16_COPY)
      return fail(CHN_ERR_OP, "gemm: preact_out is only produced by the BIAS_GELU and BF16_COPY epilogues");
    CHN_TRY(validate(preact_out, "preact_out", true));
    if (epilogue == CHN_EPI_BF16_COPY) {
      if (C->dtype != CHN_F32 || preact_out->dtype != CHN_BF16) return fail(CHN_ERR_DTYPE, "gemm: BF16_COPY needs an F32 C and a BF16 preact_out");
    } else if (preact_out->dtype != C->dtype) {
      return fail(CHN_ERR_DTYPE, "gemm: preact_out must have C's dtype");
    }
    int64_t pr, pc;
    CHN_TRY(row_major_2d(preact_out, "preact_out", &pr, &pc, &g.ldpre));
    if (pr != M || pc != N) return fail(CHN_ERR_SHAPE, "gemm: preact_out must have C's shape");
    g.pre = preact_out->data;
  }
  if (M == 0 || N == 0) return CHN_OK;
  g.A = A->data; g.B = B->data; g.C = C->data;
  g.alpha = alpha; g.beta = beta; g.epi = epilogue; g.c_bf16 = C->dtype == CHN_BF16;
  {
    const int vb = 4 * csz;  // bytes of a 4-element vector of C's dtype
    auto ok = [&](const void *q, int64_t ld) { return q == nullptr || (reinterpret_cast<uintptr_t>(q) % vb == 0 && ld % 4 == 0); };
    g.epi_vec = ok(g.C, g.ldc) && ok(g.aux, g.ldaux) && ok(g.pre, g.ldpre) &&
                (g.bias == nullptr || reinterpret_cast<uintptr_t>(g.bias) % 16 == 0);
  }
  if (want_colsum) {
    // the sums are taken per wave tile of the 256x256 kernels, unsplit, on the vector path of the epilogue
    if (!g.epi_vec || g.piece < 8) return fail(CHN_ERR_STRIDE, "gemm: row-block column sums need operands with 8-byte pieces and 16-byte aligned C and aux rows");
    plan(&g, isz, a_kc, b_kc, false, true);
  } else {
    plan(&g, isz, a_kc, b_kc, true);
  }
  if (g.splits > 1) {
    // split-K is an optimisation: without (enough, aligned) workspace the product is planned unsplit
    if (ws && reinterpret_cast<uintptr_t>(ws) % 256 == 0 && ws_bytes >= split_bytes(g)) g.partial = static_cast<float *>(ws);
    else plan(&g, isz, a_kc, b_kc, false);
  }
  g.w8 = eight_waves(g, isz, epilogue);
  hipStream_t st = as_stream(stream);
  if (A->dtype == CHN_F32) {
    if (a_kc) return b_kc ? gemm::launch_f32_kk(g, st) : gemm::launch_f32_km(g, st);
    return b_kc ? gemm::launch_f32_mk(g, st) : gemm::launch_f32_mm(g, st);
  }
  if (a_kc) return b_kc ? gemm::launch_bf16_kk(g, st) : gemm::launch_bf16_km(g, st);
  return b_kc ? gemm::launch_bf16_mk(g, st) : gemm::launch_bf16_mm(g, st);
}

}  // extern "C"
