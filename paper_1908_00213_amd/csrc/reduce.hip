// chn_reduce_axis: fold + or max over one axis (Section "Custom CUDA Kernels": the reduction kernel).
//
// The host turns (view, axis) into one of three shapes of work:
//   ROW  the reduced axis has unit stride and the kept dimensions merge into one pitched row index:
//        a group of G lanes (8 / 64 / 256) walks each row with 16-byte loads, folds through wave
//        butterflies (and LDS across the four waves of a block for G = 256);
//   COL  the innermost kept dimension has unit stride: (outer O, reduced R, inner I).  Each thread
//        owns one 16-byte column group, a block is 64 column groups x 4 row lanes, and R is split
//        over S blocks whose fp32 partial sums land in the caller's workspace and are folded by a
//        second launch of the same kernel -- no atomics, so results are bit-reproducible; a short stack
//        of rows that fits the caches (a bias gradient) is folded by one launch of tall, narrow blocks;
//   GEN  anything else: one thread per output element.
// A transposed 2-d view simply swaps ROW and COL.  HBM-bound: the input is read exactly once.
#include "common.h"

#include <mutex>

namespace chn {
namespace {

// Partial sums of chn_reduce_axis_static: one array per GPU for the life of the process.  In host code
// the name is only a handle for hipGetSymbolAddress; kernels receive the address that call returns.
constexpr size_t kScratchBytes = (size_t)CHN_REDUCE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {nullptr};
std::mutex g_scratch_mutex;

// Address of the current device's copy of `scratch` (looked up once per device, with that device current).
chn_status scratch_of_current_device(void **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(CHN_ERR_LAUNCH, "reduce (static scratch): hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(CHN_ERR_LAUNCH, "reduce (static scratch): device ordinal %d not supported", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return fail(CHN_ERR_LAUNCH, "reduce (static scratch): hipGetSymbolAddress: %s", hipGetErrorString(e));
    }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return CHN_OK;
}

template <int OP> __device__ __forceinline__ float fold(float a, float b) {
  if constexpr (OP == CHN_REDUCE_SUM) return a + b; else return fmaxf(a, b);
}
template <int OP> __device__ __forceinline__ float identity() {
  if constexpr (OP == CHN_REDUCE_SUM) return 0.0f; else return -INFINITY;
}

enum { KIND_EMPTY = 0, KIND_ROW = 1, KIND_COL = 2, KIND_GEN = 3 };

struct RPlan {
  int kind = KIND_GEN;
  int64_t len = 0, total_out = 0;
  int64_t sR = 0;            // element stride of the reduced axis
  // kept dimensions after dropping length-1 and merging
  int nk = 0;
  int64_t kshape[CHN_MAX_NDIM] = {0}, kstr[CHN_MAX_NDIM] = {0};
  // COL
  int64_t O = 1, I = 1, sO = 0;
  int split = 1;
  int64_t rows_per_split = 0;
  bool vec = false;
  int tx = 64;               // column groups per block
  size_t ws_bytes = 0;
};

// COL kernel block shapes (column groups x row lanes = 256 threads): 16 x 16 for the large streaming
// case (more column blocks, hence fewer row splits and a smaller second pass), 64 x 4 otherwise.
constexpr int kColTXWide = 16, kColTXMid = 32, kColTXNarrow = 64;
// A stack of at most kShortRows rows that fits the caches (a bias gradient: the column sums of one
// layer's output gradient) takes a single launch instead: blocks 4 column groups wide and 64 row lanes
// tall, every lane's loads (up to 16) in flight at once, so the launch lasts about one memory latency.
constexpr int kColTXShort = 4;
constexpr int64_t kShortRows = 2048, kShortBytes = 8 << 20;

chn_status make_rplan(const chn_array *in, int axis, RPlan *p) {
  CHN_TRY(validate(in, "in", false));
  if (!is_float(in->dtype)) return fail(CHN_ERR_DTYPE, "reduce: input must be F32 or BF16");
  if (in->ndim < 1) return fail(CHN_ERR_NDIM, "reduce: input needs at least one dimension");
  int ax = axis < 0 ? axis + in->ndim : axis;
  if (ax < 0 || ax >= in->ndim) return fail(CHN_ERR_AXIS, "reduce: axis %d out of range for ndim %d", axis, in->ndim);
  const int isz = dtype_size(in->dtype);
  p->len = in->shape[ax];
  p->sR = p->len > 1 ? in->strides[ax] / isz : 1;
  p->total_out = 1;
  int nk = 0;
  for (int d = 0; d < in->ndim; ++d) {
    if (d == ax) continue;
    p->total_out *= in->shape[d];
    if (in->shape[d] == 1) continue;
    p->kshape[nk] = in->shape[d];
    p->kstr[nk] = in->strides[d] / isz;
    ++nk;
  }
  if (p->total_out == 0 || p->len == 0) { p->kind = KIND_EMPTY; p->nk = nk; return CHN_OK; }
  int w = 0;
  for (int d = 1; d < nk; ++d) {
    if (p->kstr[w] == p->kstr[d] * p->kshape[d]) {
      p->kshape[w] *= p->kshape[d]; p->kstr[w] = p->kstr[d];
    } else {
      ++w; p->kshape[w] = p->kshape[d]; p->kstr[w] = p->kstr[d];
    }
  }
  nk = nk == 0 ? 0 : w + 1;
  p->nk = nk;
  if ((p->sR == 1 || p->len == 1) && nk <= 1) { p->kind = KIND_ROW; return CHN_OK; }
  if (nk >= 1 && nk <= 2 && p->kstr[nk - 1] == 1) {
    p->kind = KIND_COL;
    p->I = p->kshape[nk - 1];
    p->O = nk == 2 ? p->kshape[0] : 1;
    p->sO = nk == 2 ? p->kstr[0] : 0;
    const int n = 16 / isz;
    p->vec = reinterpret_cast<uintptr_t>(in->data) % 16 == 0 && p->I % n == 0 && p->sR % n == 0 && p->sO % n == 0;
    const int64_t groups = p->I / (p->vec ? n : 1);
    p->tx = (p->vec && groups >= 512 && p->len >= 1024) ? (isz == 2 && groups >= 1024 ? kColTXMid : kColTXWide) : kColTXNarrow;
    if (p->vec && groups >= 64 && p->len <= 64) p->tx = kColTXWide;   // 16 row lanes: one batch of loads per thread
    const int64_t cols_per_block = (int64_t)p->tx * (p->vec ? n : 1);
    const int64_t blocks_xy = ((p->I + cols_per_block - 1) / cols_per_block) * p->O;
    // Measured on 8192 x 8192: many short blocks (8 rows per thread, 16 of bf16) stream best.
    const int rpt = isz == 2 ? 16 : 8;   // rows per thread (bf16: half the partial sums for the second pass, -5 %)
    int64_t s = p->len / (rpt * (256 / p->tx));
    if (blocks_xy * s > 16384) s = 16384 / blocks_xy;
    if (p->len <= 64) s = 1;        // a short stack of rows (e.g. per-row-block sums): one launch, a few loads per thread
    if (s < 1) s = 1;
    if (s > 1024) s = 1024;
    if (s > 1 && p->len <= kShortRows && p->O * p->len * p->I * isz <= (p->vec ? kShortBytes : kShortBytes / 8)) {
      p->tx = kColTXShort;
      s = 1;
    }
    p->split = (int)s;
    p->rows_per_split = (p->len + s - 1) / s;
    p->split = (int)((p->len + p->rows_per_split - 1) / p->rows_per_split);
    p->ws_bytes = p->split > 1 ? (size_t)p->split * p->O * p->I * sizeof(float) : 0;
    return CHN_OK;
  }
  p->kind = KIND_GEN;
  return CHN_OK;
}

// ------------------------------------------------------------------------------------------------
template <typename Tout>
__global__ __launch_bounds__(256) void fill_kernel(Tout *out, int64_t n, float v) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) Elem<Tout>::store(out + i, v);
}

// ROW: G lanes per row, 256 / G rows per block.
template <int OP, typename Tin, typename Tout, int G, bool VEC>
__global__ __launch_bounds__(256) void reduce_row_kernel(const Tin *in, Tout *out, int64_t rows, int64_t len, int64_t pitch) {
  constexpr int RPB = 256 / G;
  const int g = threadIdx.x % G;
  const int64_t row = (int64_t)blockIdx.x * RPB + threadIdx.x / G;
  float acc[4] = {identity<OP>(), identity<OP>(), identity<OP>(), identity<OP>()};
  if (row < rows) {
    const Tin *p = in + row * pitch;
    if constexpr (VEC) {
      constexpr int N = Vec16<Tin>::N;
      const int64_t nvec = len / N;
      int64_t v = g;
      for (; v + 3 * G < nvec; v += 4 * G) {
        Vec16<Tin> x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) x[u].load_nt(p + (v + u * G) * N);
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int i = 0; i < N; ++i) acc[u] = fold<OP>(acc[u], x[u].get(i));
      }
      for (; v < nvec; v += G) {
        Vec16<Tin> x;
        x.load(p + v * N);
#pragma unroll
        for (int i = 0; i < N; ++i) acc[0] = fold<OP>(acc[0], x.get(i));
      }
      for (int64_t c = nvec * N + g; c < len; c += G) acc[1] = fold<OP>(acc[1], Elem<Tin>::load(p + c));
    } else {
      int64_t c = g;
      for (; c + 3 * G < len; c += 4 * G) {
        float x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) x[u] = Elem<Tin>::load(p + c + u * G);
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[u] = fold<OP>(acc[u], x[u]);
      }
      for (; c < len; c += G) acc[0] = fold<OP>(acc[0], Elem<Tin>::load(p + c));
    }
  }
  float a = fold<OP>(fold<OP>(acc[0], acc[1]), fold<OP>(acc[2], acc[3]));
  constexpr int W = G < 64 ? G : 64;
#pragma unroll
  for (int o = W / 2; o > 0; o >>= 1) a = fold<OP>(a, __shfl_xor(a, o, 64));
  if constexpr (G == 256) {
    __shared__ float part[4];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = a;
    __syncthreads();
    if (threadIdx.x == 0 && row < rows)
      Elem<Tout>::store(out + row, fold<OP>(fold<OP>(part[0], part[1]), fold<OP>(part[2], part[3])));
  } else {
    if (g == 0 && row < rows) Elem<Tout>::store(out + row, a);
  }
}

// COL: out[o, i] (or partial[s, o, i]) = fold over r in this block's slice of in[o*sO + r*sR + i].
template <int OP, typename Tin, typename Tout, bool VEC, int kColTX>
__global__ __launch_bounds__(256) void reduce_col_kernel(const Tin *in, Tout *out, int64_t R, int64_t I, int64_t sO, int64_t sR,
                                                         int64_t rows_per_split, int64_t out_split_stride) {
  constexpr int N = VEC ? Vec16<Tin>::N : 1;
  constexpr int kColTY = 256 / kColTX;
  const int tx = threadIdx.x % kColTX, ty = threadIdx.x / kColTX;
  const int64_t col = ((int64_t)blockIdx.x * kColTX + tx) * N;
  const int64_t o = blockIdx.z;
  const int64_t r_begin = (int64_t)blockIdx.y * rows_per_split;
  int64_t r_end = r_begin + rows_per_split;
  if (r_end > R) r_end = R;
  float acc[N];
#pragma unroll
  for (int i = 0; i < N; ++i) acc[i] = identity<OP>();
  if (col < I) {
    const Tin *p = in + o * sO + col;
    int64_t r = r_begin + ty;
    if constexpr (kColTX == kColTXShort) {
      constexpr int U = 16;
      for (; r < r_end; r += U * kColTY) {
        std::conditional_t<VEC, Vec16<Tin>, float> x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {          // a lane past the end re-reads its first row and drops it
          const int64_t rr = r + u * kColTY;
          const Tin *q = p + (rr < r_end ? rr : r) * sR;
          if constexpr (VEC) x[u].load(q); else x[u] = Elem<Tin>::load(q);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (r + u * kColTY < r_end) {
            if constexpr (VEC) {
#pragma unroll
              for (int i = 0; i < N; ++i) acc[i] = fold<OP>(acc[i], x[u].get(i));
            } else {
              acc[0] = fold<OP>(acc[0], x[u]);
            }
          }
      }
    } else if constexpr (VEC) {
      for (; r + 3 * kColTY < r_end; r += 4 * kColTY) {
        Vec16<Tin> x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) x[u].load_nt(p + (r + u * kColTY) * sR);
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int i = 0; i < N; ++i) acc[i] = fold<OP>(acc[i], x[u].get(i));
      }
      for (; r < r_end; r += kColTY) {
        Vec16<Tin> x;
        x.load(p + r * sR);
#pragma unroll
        for (int i = 0; i < N; ++i) acc[i] = fold<OP>(acc[i], x.get(i));
      }
    } else {
      for (; r + 3 * kColTY < r_end; r += 4 * kColTY) {
        float x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) x[u] = Elem<Tin>::load(p + (r + u * kColTY) * sR);
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[0] = fold<OP>(acc[0], x[u]);
      }
      for (; r < r_end; r += kColTY) acc[0] = fold<OP>(acc[0], Elem<Tin>::load(p + r * sR));
    }
  }
  // The short shape folds its 16 row lanes per wave with butterflies first (lanes of one column
  // group are 4 apart), so that only one partial per wave goes through LDS.
  constexpr int kParts = kColTX == kColTXShort ? 4 : kColTY;
  __shared__ float part[kParts][kColTX * N + 1];
  if constexpr (kColTX == kColTXShort) {
#pragma unroll
    for (int i = 0; i < N; ++i)
#pragma unroll
      for (int off = kColTX; off < 64; off <<= 1) acc[i] = fold<OP>(acc[i], __shfl_xor(acc[i], off));
    if (threadIdx.x % 64 < kColTX) {
#pragma unroll
      for (int i = 0; i < N; ++i) part[threadIdx.x / 64][tx * N + i] = acc[i];
    }
  } else {
#pragma unroll
    for (int i = 0; i < N; ++i) part[ty][tx * N + i] = acc[i];
  }
  __syncthreads();
  if (ty == 0 && col < I) {
    Tout *q = out + (int64_t)blockIdx.y * out_split_stride + o * I + col;
#pragma unroll
    for (int i = 0; i < N; ++i) {
      float a = part[0][tx * N + i];
#pragma unroll
      for (int y = 1; y < kParts; ++y) a = fold<OP>(a, part[y][tx * N + i]);
      Elem<Tout>::store(q + i, a);
    }
  }
}

struct GenArgs {
  int nk;
  int64_t kshape[CHN_MAX_NDIM], kstr[CHN_MAX_NDIM];
  int64_t len, sR, total_out;
};

template <int OP, typename Tin, typename Tout>
__global__ __launch_bounds__(256) void reduce_gen_kernel(const Tin *in, Tout *out, GenArgs a) {
  int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= a.total_out) return;
  int64_t off = 0, rem = e;
  for (int d = a.nk - 1; d >= 0; --d) { off += (rem % a.kshape[d]) * a.kstr[d]; rem /= a.kshape[d]; }
  float acc = identity<OP>();
  for (int64_t r = 0; r < a.len; ++r) acc = fold<OP>(acc, Elem<Tin>::load(in + off + r * a.sR));
  Elem<Tout>::store(out + e, acc);
}

template <int OP, typename Tin, typename Tout>
chn_status launch_col(const Tin *in, Tout *out, const RPlan &p, int64_t O, int64_t R, int64_t I, int64_t sO, int64_t sR,
                      int split, int64_t rps, int64_t split_stride, bool vec, int tx, hipStream_t st) {
  if (!vec && tx != kColTXShort) tx = kColTXNarrow;
  const int n = vec ? 16 / (int)sizeof(Tin) : 1;
  const int64_t cpb = (int64_t)tx * n;
  dim3 grid((unsigned)((I + cpb - 1) / cpb), (unsigned)split, (unsigned)O);
  if (O > 65535) return fail(CHN_ERR_SHAPE, "reduce: outer extent %lld too large for the column kernel", (long long)O);
  if (vec && tx == kColTXShort) hipLaunchKernelGGL((reduce_col_kernel<OP, Tin, Tout, true, kColTXShort>), grid, dim3(256), 0, st, in, out, R, I, sO, sR, rps, split_stride);
  else if (vec && tx == kColTXWide) hipLaunchKernelGGL((reduce_col_kernel<OP, Tin, Tout, true, kColTXWide>), grid, dim3(256), 0, st, in, out, R, I, sO, sR, rps, split_stride);
  else if (vec && tx == kColTXMid) hipLaunchKernelGGL((reduce_col_kernel<OP, Tin, Tout, true, kColTXMid>), grid, dim3(256), 0, st, in, out, R, I, sO, sR, rps, split_stride);
  else if (vec) hipLaunchKernelGGL((reduce_col_kernel<OP, Tin, Tout, true, kColTXNarrow>), grid, dim3(256), 0, st, in, out, R, I, sO, sR, rps, split_stride);
  else if (tx == kColTXShort) hipLaunchKernelGGL((reduce_col_kernel<OP, Tin, Tout, false, kColTXShort>), grid, dim3(256), 0, st, in, out, R, I, sO, sR, rps, split_stride);
  else hipLaunchKernelGGL((reduce_col_kernel<OP, Tin, Tout, false, kColTXNarrow>), grid, dim3(256), 0, st, in, out, R, I, sO, sR, rps, split_stride);
  (void)p;
  return check_launch("reduce col");
}

template <int OP, typename Tin, typename Tout>
chn_status launch(const RPlan &p, const chn_array *in, const chn_array *out, void *ws, hipStream_t st) {
  const Tin *src = static_cast<const Tin *>(in->data);
  Tout *dst = static_cast<Tout *>(out->data);
  if (p.kind == KIND_ROW) {
    const int64_t rows = p.nk == 1 ? p.kshape[0] : 1;
    const int64_t pitch = p.nk == 1 ? p.kstr[0] : 0;
    const int n = 16 / (int)sizeof(Tin);
    const bool vec = reinterpret_cast<uintptr_t>(src) % 16 == 0 && pitch % n == 0 && p.len >= 4 * n;
#define CHN_ROW(G)                                                                                          \
  do {                                                                                                      \
    const int64_t blocks = (rows + (256 / G) - 1) / (256 / G);                                              \
    if (blocks > 0x7fffffff) return fail(CHN_ERR_SHAPE, "reduce: too many rows");                           \
    if (vec) hipLaunchKernelGGL((reduce_row_kernel<OP, Tin, Tout, G, true>), dim3((unsigned)blocks), dim3(256), 0, st, src, dst, rows, p.len, pitch); \
    else hipLaunchKernelGGL((reduce_row_kernel<OP, Tin, Tout, G, false>), dim3((unsigned)blocks), dim3(256), 0, st, src, dst, rows, p.len, pitch);    \
  } while (0)
    if (p.len >= 2048 || rows < 512) CHN_ROW(256);
    else if (p.len > 64) CHN_ROW(64);
    else CHN_ROW(8);
#undef CHN_ROW
    return check_launch("reduce row");
  }
  if (p.kind == KIND_COL) {
    if (p.split == 1)
      return launch_col<OP, Tin, Tout>(src, dst, p, p.O, p.len, p.I, p.sO, p.sR, 1, p.len, 0, p.vec, p.tx, st);
    float *part = static_cast<float *>(ws);
    const int64_t OI = p.O * p.I;
    CHN_TRY((launch_col<OP, Tin, float>(src, part, p, p.O, p.len, p.I, p.sO, p.sR, p.split, p.rows_per_split, OI, p.vec, p.tx, st)));
    // Second pass over the [split, O * I] partials: a small array, so the time is one chain of
    // dependent load batches per lane; the narrow-in-columns block shape keeps that chain short.
    const bool wide2 = OI % 4 == 0 && OI / 4 >= 512 && p.split >= 16;
    return launch_col<OP, float, Tout>(part, dst, p, 1, p.split, OI, 0, OI, 1, p.split, 0, OI % 4 == 0, wide2 ? kColTXWide : kColTXNarrow, st);
  }
  GenArgs a{};
  a.nk = p.nk; a.len = p.len; a.sR = p.sR; a.total_out = p.total_out;
  for (int d = 0; d < p.nk; ++d) { a.kshape[d] = p.kshape[d]; a.kstr[d] = p.kstr[d]; }
  const int64_t blocks = (p.total_out + 255) / 256;
  if (blocks > 0x7fffffff) return fail(CHN_ERR_SHAPE, "reduce: output too large");
  hipLaunchKernelGGL((reduce_gen_kernel<OP, Tin, Tout>), dim3((unsigned)blocks), dim3(256), 0, st, src, dst, a);
  return check_launch("reduce general");
}

template <typename Tin, typename Tout>
chn_status launch_op(int op, const RPlan &p, const chn_array *in, const chn_array *out, void *ws, hipStream_t st) {
  if (op == CHN_REDUCE_SUM) return launch<CHN_REDUCE_SUM, Tin, Tout>(p, in, out, ws, st);
  return launch<CHN_REDUCE_MAX, Tin, Tout>(p, in, out, ws, st);
}

}  // namespace

chn_status reduce_one_axis(int op, const chn_array *in, int axis, int keepdims, const chn_array *out,
                           void *ws, size_t ws_bytes, bool static_scratch, chn_stream stream) {
  if (op != CHN_REDUCE_SUM && op != CHN_REDUCE_MAX) return fail(CHN_ERR_OP, "reduce: unknown op %d", op);
  RPlan p;
  CHN_TRY(make_rplan(in, axis, &p));
  CHN_TRY(validate(out, "out", true));
  if (!is_float(out->dtype)) return fail(CHN_ERR_DTYPE, "reduce: out must be F32 or BF16");
  const int ax = axis < 0 ? axis + in->ndim : axis;
  const int ond = keepdims ? in->ndim : in->ndim - 1;
  if (out->ndim != ond) return fail(CHN_ERR_SHAPE, "reduce: out has ndim %d, expected %d", out->ndim, ond);
  for (int d = 0, od = 0; d < in->ndim; ++d) {
    if (d == ax) {
      if (keepdims) { if (out->shape[od] != 1) return fail(CHN_ERR_SHAPE, "reduce: kept axis must have length 1"); ++od; }
      continue;
    }
    if (out->shape[od] != in->shape[d]) return fail(CHN_ERR_SHAPE, "reduce: out dimension %d has length %lld, expected %lld", od, (long long)out->shape[od], (long long)in->shape[d]);
    ++od;
  }
  if (!is_contiguous(out)) return fail(CHN_ERR_STRIDE, "reduce: out must be contiguous");
  if (p.total_out == 0) return CHN_OK;
  hipStream_t st = as_stream(stream);
  if (p.kind == KIND_EMPTY) {
    const float v = op == CHN_REDUCE_SUM ? 0.0f : -INFINITY;
    const unsigned blocks = (unsigned)((p.total_out + 255) / 256);
    if (out->dtype == CHN_F32) hipLaunchKernelGGL((fill_kernel<float>), dim3(blocks), dim3(256), 0, st, static_cast<float *>(out->data), p.total_out, v);
    else hipLaunchKernelGGL((fill_kernel<bf16_raw>), dim3(blocks), dim3(256), 0, st, static_cast<bf16_raw *>(out->data), p.total_out, v);
    return check_launch("reduce fill");
  }
  if (p.kind == KIND_COL && p.ws_bytes > 0) {
    if (static_scratch) {
      // the per-device array stands in for the caller's workspace; nothing is allocated
      if (p.ws_bytes > kScratchBytes)
        return fail(CHN_ERR_WORKSPACE, "reduce (static scratch): this reduction needs %zu bytes of partial sums, the built-in buffer holds %zu; use chn_reduce_axis with a workspace",
                    p.ws_bytes, kScratchBytes);
      CHN_TRY(scratch_of_current_device(&ws));
    } else {
      CHN_TRY(check_ws(ws, ws_bytes, p.ws_bytes, "reduce"));
    }
  }
  if (in->dtype == CHN_F32 && out->dtype == CHN_F32) return launch_op<float, float>(op, p, in, out, ws, st);
  if (in->dtype == CHN_BF16 && out->dtype == CHN_F32) return launch_op<bf16_raw, float>(op, p, in, out, ws, st);
  if (in->dtype == CHN_BF16 && out->dtype == CHN_BF16) return launch_op<bf16_raw, bf16_raw>(op, p, in, out, ws, st);
  return launch_op<float, bf16_raw>(op, p, in, out, ws, st);
}

// ---- several axes at once ---------------------------------------------------------------------------------
// CHN_AXES(mask) / CHN_AXIS_ALL are carried out as a sequence of single-axis reductions, last axis first,
// over fp32 intermediates in the caller's workspace: neighbouring reduced dimensions that are jointly
// contiguous are merged into one axis first (a full sum of a contiguous array is one axis), and an axis that
// is folded into very few results is cut in two (length = r x c: c elements per row first, then the r row
// results), because a single-axis reduction gives every result to one workgroup.
struct Pass {
  chn_array in, out;     // out: contiguous fp32 intermediate, or the caller's out for the last pass
  int axis;
  size_t ws_need;        // partial sums of the column kernel for this pass
};
struct MultiPlan {
  Pass pass[2 * CHN_MAX_NDIM];
  int n = 0;
  size_t tmp_bytes[2] = {0, 0};   // two intermediates that take turns
  size_t partial_bytes = 0;
  size_t total() const { return ((tmp_bytes[0] + 255) & ~size_t(255)) + ((tmp_bytes[1] + 255) & ~size_t(255)) + partial_bytes; }
};

void set_contiguous(chn_array *a, int dtype) {
  int64_t st = dtype_size(dtype);
  a->dtype = dtype;
  for (int d = a->ndim - 1; d >= 0; --d) { a->strides[d] = st; st *= a->shape[d] > 0 ? a->shape[d] : 1; }
}

chn_status make_multi(const chn_array *in, int axis_code, MultiPlan *mp) {
  CHN_TRY(validate(in, "in", false));
  if (!is_float(in->dtype)) return fail(CHN_ERR_DTYPE, "reduce: input must be F32 or BF16");
  const int nd = in->ndim;
  if (nd < 1) return fail(CHN_ERR_NDIM, "reduce: input needs at least one dimension");
  int mask;
  if (axis_code == CHN_AXIS_ALL) mask = (1 << nd) - 1;
  else {
    mask = axis_code - CHN_AXES(0);
    if (mask <= 0 || (mask >> nd) != 0) return fail(CHN_ERR_AXIS, "reduce: axis set 0x%x out of range for %d dimensions", mask, nd);
  }
  // working copy of the view; reduced flag per dimension
  chn_array cur = *in;
  bool red[CHN_MAX_NDIM];
  for (int d = 0; d < nd; ++d) red[d] = (mask >> d) & 1;
  // merge neighbouring reduced dimensions that are jointly contiguous (or of length 1)
  for (int d = cur.ndim - 2; d >= 0; --d) {
    if (!(red[d] && red[d + 1])) continue;
    const bool joint = cur.shape[d + 1] == 1 || cur.shape[d] == 1 || cur.strides[d] == cur.strides[d + 1] * cur.shape[d + 1];
    if (!joint) continue;
    if (cur.shape[d + 1] == 1) cur.strides[d + 1] = cur.strides[d];     // keep the stride that matters
    cur.shape[d + 1] *= cur.shape[d];
    for (int e = d; e + 1 < cur.ndim; ++e) { cur.shape[e] = cur.shape[e + 1]; cur.strides[e] = cur.strides[e + 1]; red[e] = red[e + 1]; }
    --cur.ndim;
  }
  int64_t kept = 1;
  for (int d = 0; d < cur.ndim; ++d) if (!red[d]) kept *= cur.shape[d];
  // cut a long axis with few results in two: (.., L, ..) -> (.., r, c, ..), both reduced
  for (int d = 0; d < cur.ndim && cur.ndim < CHN_MAX_NDIM; ++d) {
    if (!red[d] || cur.shape[d] < (1 << 20) || kept >= 512) continue;
    int64_t c = 0;
    for (int64_t t = 8192; t >= 1024; t -= 4) if (cur.shape[d] % t == 0) { c = t; break; }
    if (!c) continue;
    for (int e = cur.ndim; e > d + 1; --e) { cur.shape[e] = cur.shape[e - 1]; cur.strides[e] = cur.strides[e - 1]; red[e] = red[e - 1]; }
    ++cur.ndim;
    cur.shape[d + 1] = c; cur.strides[d + 1] = cur.strides[d]; red[d + 1] = true;
    cur.shape[d] /= c; cur.strides[d] = cur.strides[d + 1] * c;
    ++d;
  }
  // one pass per remaining reduced dimension, last first
  int which = 0;
  for (int d = cur.ndim - 1; d >= 0; --d) {
    if (!red[d]) continue;
    Pass &ps = mp->pass[mp->n++];
    ps.in = cur;
    ps.axis = d;
    chn_array nxt = cur;
    for (int e = d; e + 1 < nxt.ndim; ++e) { nxt.shape[e] = nxt.shape[e + 1]; red[e] = red[e + 1]; }
    --nxt.ndim;
    set_contiguous(&nxt, CHN_F32);
    nxt.data = nullptr;                      // filled in when the workspace is known
    ps.out = nxt;
    RPlan rp;
    chn_array probe = ps.in;
    if (!probe.data) probe.data = reinterpret_cast<void *>(uintptr_t(256));   // (planning only looks at alignment)
    CHN_TRY(make_rplan(&probe, d, &rp));
    ps.ws_need = rp.kind == KIND_COL ? rp.ws_bytes : 0;
    if (ps.ws_need > mp->partial_bytes) mp->partial_bytes = ps.ws_need;
    const size_t ob = (size_t)numel(&nxt) * sizeof(float);
    if (ob > mp->tmp_bytes[which]) mp->tmp_bytes[which] = ob;
    which ^= 1;
    cur = nxt;
  }
  return CHN_OK;
}

chn_status reduce_axis_impl(int op, const chn_array *in, int axis, int keepdims, const chn_array *out,
                            void *ws, size_t ws_bytes, bool static_scratch, chn_stream stream) {
  if (axis != CHN_AXIS_ALL && axis < CHN_AXES(0)) return reduce_one_axis(op, in, axis, keepdims, out, ws, ws_bytes, static_scratch, stream);
  if (op != CHN_REDUCE_SUM && op != CHN_REDUCE_MAX) return fail(CHN_ERR_OP, "reduce: unknown op %d", op);
  MultiPlan mp;
  CHN_TRY(make_multi(in, axis, &mp));
  CHN_TRY(validate(out, "out", true));
  if (!is_float(out->dtype)) return fail(CHN_ERR_DTYPE, "reduce: out must be F32 or BF16");
  if (!is_contiguous(out)) return fail(CHN_ERR_STRIDE, "reduce: out must be contiguous");
  // expected shape of out
  const int nd = in->ndim;
  const int mask = axis == CHN_AXIS_ALL ? (1 << nd) - 1 : axis - CHN_AXES(0);
  int od = 0;
  for (int d = 0; d < nd; ++d) {
    const bool r = (mask >> d) & 1;
    if (r && !keepdims) continue;
    if (od >= out->ndim || out->shape[od] != (r ? 1 : in->shape[d]))
      return fail(CHN_ERR_SHAPE, "reduce: out dimension %d does not match the reduced shape", od);
    ++od;
  }
  if (od != out->ndim) return fail(CHN_ERR_SHAPE, "reduce: out has ndim %d, expected %d", out->ndim, od);
  if (numel(out) == 0) return CHN_OK;
  const size_t need = static_scratch ? 0 : mp.total();
  if (static_scratch) {
    if (mp.total() > kScratchBytes)
      return fail(CHN_ERR_WORKSPACE, "reduce (static scratch): this reduction needs %zu bytes of intermediates, the built-in buffer holds %zu; use chn_reduce_axis with a workspace",
                  mp.total(), kScratchBytes);
    if (mp.total() > 0) CHN_TRY(scratch_of_current_device(&ws));
  } else {
    CHN_TRY(check_ws(ws, ws_bytes, need, "reduce"));
  }
  char *base = static_cast<char *>(ws);
  char *tmp[2] = {base, base ? base + ((mp.tmp_bytes[0] + 255) & ~size_t(255)) : nullptr};
  char *partial = base ? tmp[1] + ((mp.tmp_bytes[1] + 255) & ~size_t(255)) : nullptr;
  const void *src = in->data;
  for (int i = 0; i < mp.n; ++i) {
    Pass &ps = mp.pass[i];
    ps.in.data = const_cast<void *>(src);
    const bool last = i == mp.n - 1;
    if (last) { ps.out.data = out->data; set_contiguous(&ps.out, out->dtype); }
    else ps.out.data = tmp[i & 1];
    CHN_TRY(reduce_one_axis(op, &ps.in, ps.axis, 0, &ps.out, partial, mp.partial_bytes, false, stream));
    src = ps.out.data;
  }
  return CHN_OK;
}


}  // namespace chn

extern "C" {

size_t chn_reduce_axis_workspace_bytes(const chn_array *in, int axis) {
  if (axis == CHN_AXIS_ALL || axis >= CHN_AXES(0)) {
    chn::MultiPlan mp;
    if (!in || chn::make_multi(in, axis, &mp) != CHN_OK) return 0;
    return mp.total();
  }
  chn::RPlan p;
  if (chn::make_rplan(in, axis, &p) != CHN_OK) return 0;
  return p.kind == chn::KIND_COL ? p.ws_bytes : 0;
}

chn_status chn_reduce_axis(int op, const chn_array *in, int axis, int keepdims, const chn_array *out,
                           void *ws, size_t ws_bytes, chn_stream stream) {
  return chn::reduce_axis_impl(op, in, axis, keepdims, out, ws, ws_bytes, false, stream);
}

chn_status chn_reduce_axis_static(int op, const chn_array *in, int axis, int keepdims, const chn_array *out,
                                  chn_stream stream) {
  return chn::reduce_axis_impl(op, in, axis, keepdims, out, nullptr, 0, true, stream);
}

}  // extern "C"
