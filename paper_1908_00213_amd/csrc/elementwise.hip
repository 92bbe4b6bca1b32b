// chn_elementwise_broadcast: NumPy-broadcast element-wise maps (Section "Custom CUDA Kernels" of the
// paper: the element-wise kernel; figure "Example of a user-defined kernel": w = x*y + z).
//
// The host resolves broadcasting into per-operand element strides, drops length-1 dimensions, orders
// the dimensions by the output's stride, merges neighbours that are jointly contiguous in every
// operand, and then picks one of four kernel families:
//   0  flat      output and full-size inputs contiguous; other inputs repeat with a fixed period
//                (row broadcast, e.g. a bias) or are scalars.  16-byte vector loads and stores.
//   1  rows      every operand has inner stride 1 or 0; outer dimensions arbitrary (pitched rows,
//                column broadcast, sliced views).  Coalesced scalar accesses.
//   2  transpose 2-d; some inputs are unit-stride along dimension 0 (transposed views).  Those go
//                through a 64x64 LDS tile so that both their reads and the output writes coalesce.
//   3  general   anything else: one thread per element, full index decomposition.
// HBM-bound: 16-byte accesses per lane, several independent loads in flight per thread, more
// workgroups than the 256 compute units can hold at once.
#include <type_traits>

#include "common.h"

namespace chn {
namespace {

constexpr int kArity[CHN_OP_COUNT_] = {1, 2, 2, 2, 3, 3, 1, 2, 1, 2, 1, 2, 2, 2, 0, 1, 1, 1, 1, 2};
constexpr int kScalars[CHN_OP_COUNT_] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 1, 1, 0, 0, 1, 0, 0, 0, 0, 0};

// LOWP: the result is stored as bfloat16.  gelu and its derivative then use the compact forms of the
// GEMM epilogues: absolute error 1.5e-7 in Phi, so |error| <= 1.5e-7 |x|; what is lost against the
// library's erfc form is the relative accuracy far out in the negative tail, where the result is
// below 1e-5 in magnitude.  A quarter of the instructions: with erfc these ops are bound by
// arithmetic, not by HBM.
template <int OP, bool LOWP = false>
__device__ __forceinline__ float ew_apply(float x, float y, float z, float s) {
  if constexpr (LOWP && OP == CHN_OP_GELU) return gelu_epi_f(x);
  else if constexpr (LOWP && OP == CHN_OP_GELU_BWD) return x * gelu_grad_epi_f(y);
  else if constexpr (LOWP && OP == CHN_OP_ADD_GELU) return gelu_epi_f(x + y);
  else
  if constexpr (OP == CHN_OP_COPY) return x;
  else if constexpr (OP == CHN_OP_ADD) return x + y;
  else if constexpr (OP == CHN_OP_SUB) return x - y;
  else if constexpr (OP == CHN_OP_MUL) return x * y;
  else if constexpr (OP == CHN_OP_MAD) return fmaf(x, y, z);
  else if constexpr (OP == CHN_OP_MAD_RELU) return fmaxf(fmaf(x, y, z), 0.0f);
  else if constexpr (OP == CHN_OP_RELU) return fmaxf(x, 0.0f);
  else if constexpr (OP == CHN_OP_RELU_BWD) return y > 0.0f ? x : 0.0f;
  else if constexpr (OP == CHN_OP_GELU) return gelu_f(x);
  else if constexpr (OP == CHN_OP_GELU_BWD) return x * gelu_grad_f(y);
  else if constexpr (OP == CHN_OP_SCALE) return s * x;
  else if constexpr (OP == CHN_OP_AXPY) return fmaf(s, y, x);
  else if constexpr (OP == CHN_OP_ADD_RELU) return fmaxf(x + y, 0.0f);
  else if constexpr (OP == CHN_OP_ADD_GELU) return gelu_f(x + y);
  else if constexpr (OP == CHN_OP_FILL) return s;
  else if constexpr (OP == CHN_OP_SIGMOID) return sigmoid_f(x);
  else if constexpr (OP == CHN_OP_TANH) return tanhf(x);
  else if constexpr (OP == CHN_OP_SQRT) return sqrtf(x);
  else if constexpr (OP == CHN_OP_EXP) return expf(x);
  else if constexpr (OP == CHN_OP_GELU_BWD2) return x * (0.39894228040143267794f * expf(-0.5f * y * y)) * (2.0f - y * y);
  else return 0.0f;
}

template <bool LOWP = false>
__device__ __forceinline__ float ew_apply_rt(int op, float x, float y, float z, float s) {
  switch (op) {
#define CHN_CASE(OPC) case OPC: return ew_apply<OPC, LOWP>(x, y, z, s);
    CHN_CASE(CHN_OP_COPY) CHN_CASE(CHN_OP_ADD) CHN_CASE(CHN_OP_SUB) CHN_CASE(CHN_OP_MUL)
    CHN_CASE(CHN_OP_MAD) CHN_CASE(CHN_OP_MAD_RELU) CHN_CASE(CHN_OP_RELU) CHN_CASE(CHN_OP_RELU_BWD)
    CHN_CASE(CHN_OP_GELU) CHN_CASE(CHN_OP_GELU_BWD) CHN_CASE(CHN_OP_SCALE) CHN_CASE(CHN_OP_AXPY)
    CHN_CASE(CHN_OP_ADD_RELU) CHN_CASE(CHN_OP_ADD_GELU) CHN_CASE(CHN_OP_FILL)
    CHN_CASE(CHN_OP_SIGMOID) CHN_CASE(CHN_OP_TANH) CHN_CASE(CHN_OP_SQRT) CHN_CASE(CHN_OP_EXP) CHN_CASE(CHN_OP_GELU_BWD2)
#undef CHN_CASE
  }
  return 0.0f;
}

// ------------------------------------------------------------------------------------------------
// host-side plan
enum { MODE_FULL = 0, MODE_PERIODIC = 1, MODE_SCALAR = 2 };

struct Plan {
  int family = 3;
  int nd = 0;
  int n_in = 0;
  int64_t total = 0;
  int64_t shape[CHN_MAX_NDIM] = {0};
  int64_t ostr[CHN_MAX_NDIM] = {0};      // element strides
  int64_t istr[3][CHN_MAX_NDIM] = {{0}};
  int mode[3] = {0, 0, 0};               // family 0
  int64_t period[3] = {1, 1, 1};
  bool transposed[3] = {false, false, false};  // family 2
  bool tvec = false;                           // family 2: every operand allows 16-byte accesses
};

chn_status make_plan(int op, int n_in, const chn_array *const *in, const chn_array *out, Plan *p) {
  if (op < 0 || op >= CHN_OP_COUNT_) return fail(CHN_ERR_OP, "elementwise: unknown op %d", op);
  if (n_in != kArity[op]) return fail(CHN_ERR_OP, "elementwise: op %d takes %d inputs, got %d", op, kArity[op], n_in);
  if (n_in > 0 && !in) return fail(CHN_ERR_NULL, "elementwise: input list is NULL");
  CHN_TRY(validate(out, "out", true));
  if (!is_float(out->dtype)) return fail(CHN_ERR_DTYPE, "elementwise: out must be F32 or BF16");
  for (int k = 0; k < n_in; ++k) {
    CHN_TRY(validate(in[k], "in", false));
    if (!is_float(in[k]->dtype)) return fail(CHN_ERR_DTYPE, "elementwise: inputs must be F32 or BF16");
    if (in[k]->dtype != in[0]->dtype) return fail(CHN_ERR_DTYPE, "elementwise: inputs must share one dtype");
    if (in[k]->ndim > out->ndim) return fail(CHN_ERR_SHAPE, "elementwise: input %d has more dimensions than out", k);
  }
  p->n_in = n_in;
  int nd = out->ndim;
  int osz = dtype_size(out->dtype);
  int64_t shape[CHN_MAX_NDIM], ostr[CHN_MAX_NDIM], istr[3][CHN_MAX_NDIM];
  for (int d = 0; d < nd; ++d) {
    shape[d] = out->shape[d];
    ostr[d] = out->strides[d] / osz;
  }
  for (int k = 0; k < n_in; ++k) {
    int isz = dtype_size(in[k]->dtype);
    int shift = nd - in[k]->ndim;
    for (int d = 0; d < nd; ++d) {
      int id = d - shift;
      if (id < 0 || in[k]->shape[id] == 1) { istr[k][d] = 0; continue; }
      if (in[k]->shape[id] != shape[d])
        return fail(CHN_ERR_SHAPE, "elementwise: input %d has length %lld along out dimension %d of length %lld", k, (long long)in[k]->shape[id], d, (long long)shape[d]);
      istr[k][d] = in[k]->strides[id] / isz;
    }
  }
  p->total = numel(out);
  if (p->total == 0) { p->nd = 0; p->family = 0; return CHN_OK; }
  // drop length-1 dimensions
  int m = 0;
  for (int d = 0; d < nd; ++d) {
    if (shape[d] == 1) continue;
    shape[m] = shape[d]; ostr[m] = ostr[d];
    for (int k = 0; k < n_in; ++k) istr[k][m] = istr[k][d];
    ++m;
  }
  nd = m;
  // order by decreasing output stride (stable insertion sort)
  for (int i = 1; i < nd; ++i)
    for (int j = i; j > 0 && ostr[j - 1] < ostr[j]; --j) {
      std::swap(shape[j - 1], shape[j]); std::swap(ostr[j - 1], ostr[j]);
      for (int k = 0; k < n_in; ++k) std::swap(istr[k][j - 1], istr[k][j]);
    }
  // merge neighbours that are jointly contiguous in every operand
  int w = 0;
  for (int d = 1; d < nd; ++d) {
    bool ok = ostr[w] == ostr[d] * shape[d];
    for (int k = 0; k < n_in && ok; ++k) ok = istr[k][w] == istr[k][d] * shape[d];
    if (ok) {
      shape[w] *= shape[d]; ostr[w] = ostr[d];
      for (int k = 0; k < n_in; ++k) istr[k][w] = istr[k][d];
    } else {
      ++w;
      shape[w] = shape[d]; ostr[w] = ostr[d];
      for (int k = 0; k < n_in; ++k) istr[k][w] = istr[k][d];
    }
  }
  nd = nd == 0 ? 0 : w + 1;
  if (nd == 0) { nd = 1; shape[0] = 1; ostr[0] = 1; for (int k = 0; k < n_in; ++k) istr[k][0] = 0; }
  p->nd = nd;
  for (int d = 0; d < nd; ++d) {
    p->shape[d] = shape[d]; p->ostr[d] = ostr[d];
    for (int k = 0; k < n_in; ++k) p->istr[k][d] = istr[k][d];
  }
  // classify
  const int last = nd - 1;
  bool out_inner_unit = ostr[last] == 1 || shape[last] == 1;
  bool inner_01 = out_inner_unit;
  for (int k = 0; k < n_in; ++k) inner_01 = inner_01 && (istr[k][last] == 1 || istr[k][last] == 0);
  auto aligned16 = [](const void *q) { return reinterpret_cast<uintptr_t>(q) % 16 == 0; };
  bool ptrs16 = aligned16(out->data);
  for (int k = 0; k < n_in; ++k) ptrs16 = ptrs16 && aligned16(in[k]->data);
  if (inner_01 && ptrs16 && nd <= 2) {
    bool ok = nd == 1 || ostr[0] == shape[1];
    for (int k = 0; k < n_in && ok; ++k) {
      if (nd == 1) {
        p->mode[k] = istr[k][0] == 1 ? MODE_FULL : MODE_SCALAR;
      } else if (istr[k][1] == 1 && istr[k][0] == shape[1]) {
        p->mode[k] = MODE_FULL;
      } else if (istr[k][1] == 1 && istr[k][0] == 0) {
        p->mode[k] = MODE_PERIODIC; p->period[k] = shape[1];
      } else if (istr[k][1] == 0 && istr[k][0] == 0) {
        p->mode[k] = MODE_SCALAR;
      } else {
        ok = false;
      }
    }
    if (ok) { p->family = 0; return CHN_OK; }
  }
  if (inner_01) { p->family = 1; return CHN_OK; }
  if (nd == 2 && out_inner_unit) {
    bool ok = true, any = false;
    for (int k = 0; k < n_in; ++k) {
      if (istr[k][1] == 1 || istr[k][1] == 0) { p->transposed[k] = false; continue; }
      if (istr[k][0] == 1) { p->transposed[k] = true; any = true; continue; }
      ok = false;
    }
    if (ok && any) {
      p->family = 2;
      // vector form: one dtype, extents and strides in whole 16-byte vectors, 16-byte aligned bases
      const int e = 16 / osz;
      bool v = n_in > 0 && in[0]->dtype == out->dtype && shape[0] % e == 0 && shape[1] % e == 0 &&
               aligned16(out->data) && ostr[0] % e == 0;
      for (int k = 0; k < n_in && v; ++k) {
        if (p->transposed[k]) v = aligned16(in[k]->data) && istr[k][1] % e == 0;
        else if (istr[k][1] == 1) v = aligned16(in[k]->data) && istr[k][0] % e == 0;
      }
      p->tvec = v;
      return CHN_OK;
    }
  }
  p->family = 3;
  return CHN_OK;
}

// ------------------------------------------------------------------------------------------------
// family 0: flat vector kernel
struct FlatArgs {
  const void *in[3];
  void *out;
  int64_t total;
  int64_t period[3];
  int mode[3];
  float s0;
};

constexpr int kFlatThreads = 256;
constexpr int kFlatUnroll = 1;   // measured: one 16-byte vector per thread and a huge grid streams fastest

template <typename T, int E>
struct Pack {  // E fp32 lanes backed by 16-byte vectors of T
  static constexpr int NV = E / Vec16<T>::N;
  Vec16<T> v[NV];
  __device__ __forceinline__ void load(const T *p) {
#pragma unroll
    for (int i = 0; i < NV; ++i) v[i].load(p + i * Vec16<T>::N);
  }
  __device__ __forceinline__ void load_nt(const T *p) {
#pragma unroll
    for (int i = 0; i < NV; ++i) v[i].load_nt(p + i * Vec16<T>::N);
  }
  __device__ __forceinline__ void store_nt(T *p) const {
#pragma unroll
    for (int i = 0; i < NV; ++i) v[i].store_nt(p + i * Vec16<T>::N);
  }
  __device__ __forceinline__ float get(int i) const { return v[i / Vec16<T>::N].get(i % Vec16<T>::N); }
  __device__ __forceinline__ void set(int i, float x) { v[i / Vec16<T>::N].set(i % Vec16<T>::N, x); }
};

template <int OP, typename Tin, typename Tout, int NIN>
__global__ __launch_bounds__(kFlatThreads) void ew_flat_kernel(FlatArgs a) {
  constexpr int E = (sizeof(Tin) == 2 || sizeof(Tout) == 2) ? 8 : 4;  // elements per thread step
  const int64_t nvec = a.total / E;
  const int64_t base = (int64_t)blockIdx.x * (kFlatThreads * kFlatUnroll) + threadIdx.x;
  Pack<Tin, E> x[kFlatUnroll][NIN > 0 ? NIN : 1];
  float sc[NIN > 0 ? NIN : 1];
#pragma unroll
  for (int k = 0; k < NIN; ++k)
    sc[k] = a.mode[k] == MODE_SCALAR ? Elem<Tin>::load(static_cast<const Tin *>(a.in[k])) : 0.0f;
#pragma unroll
  for (int u = 0; u < kFlatUnroll; ++u) {
    const int64_t v = base + (int64_t)u * kFlatThreads;
    if (v < nvec) {
#pragma unroll
      for (int k = 0; k < NIN; ++k) {
        const Tin *p = static_cast<const Tin *>(a.in[k]);
        if (a.mode[k] == MODE_FULL) {
          x[u][k].load_nt(p + v * E);
        } else if (a.mode[k] == MODE_PERIODIC) {
          // 32-bit remainder when the index fits: 64-bit division is a long instruction sequence
          const int64_t off = a.total <= 0xffffffffll
                                  ? (int64_t)((uint32_t)(v * E) % (uint32_t)a.period[k])
                                  : (v * E) % a.period[k];
          if (a.period[k] % E == 0) {
            x[u][k].load(p + off);
          } else {
#pragma unroll
            for (int i = 0; i < E; ++i) x[u][k].set(i, Elem<Tin>::load(p + (off + i) % a.period[k]));
          }
        }
      }
    }
  }
#pragma unroll
  for (int u = 0; u < kFlatUnroll; ++u) {
    const int64_t v = base + (int64_t)u * kFlatThreads;
    if (v < nvec) {
      Pack<Tout, E> r;
#pragma unroll
      for (int i = 0; i < E; ++i) {
        float f[3] = {0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int k = 0; k < NIN; ++k) f[k] = a.mode[k] == MODE_SCALAR ? sc[k] : x[u][k].get(i);
        r.set(i, ew_apply<OP, sizeof(Tout) == 2>(f[0], f[1], f[2], a.s0));
      }
      r.store_nt(static_cast<Tout *>(a.out) + v * E);
    }
  }
  // ragged tail (fewer than E elements), handled by the first threads of block 0
  if (blockIdx.x == 0) {
    const int64_t e = nvec * E + threadIdx.x;
    if (e < a.total) {
      float f[3] = {0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int k = 0; k < NIN; ++k) {
        const Tin *p = static_cast<const Tin *>(a.in[k]);
        f[k] = a.mode[k] == MODE_SCALAR ? sc[k]
               : a.mode[k] == MODE_FULL ? Elem<Tin>::load(p + e) : Elem<Tin>::load(p + e % a.period[k]);
      }
      Elem<Tout>::store(static_cast<Tout *>(a.out) + e, ew_apply<OP, sizeof(Tout) == 2>(f[0], f[1], f[2], a.s0));
    }
  }
}

// ------------------------------------------------------------------------------------------------
// families 1 and 3 share the strided argument block
struct StridedArgs {
  const void *in[3];
  void *out;
  int nd;
  int n_in;
  int op;
  float s0;
  int64_t total;
  int64_t shape[CHN_MAX_NDIM];
  int64_t ostr[CHN_MAX_NDIM];
  int64_t istr[3][CHN_MAX_NDIM];
};

constexpr int kRowsThreads = 256;
constexpr int kRowsUnroll = 4;

// family 1: inner dimension has stride 1 or 0 in every operand; one block covers a chunk of one row
template <typename Tin, typename Tout>
__global__ __launch_bounds__(kRowsThreads) void ew_rows_kernel(StridedArgs a, int64_t chunks_per_row) {
  const int last = a.nd - 1;
  const int64_t n = a.shape[last];
  int64_t row = (int64_t)blockIdx.x / chunks_per_row;
  const int64_t chunk = (int64_t)blockIdx.x % chunks_per_row;
  int64_t ooff = 0, ioff[3] = {0, 0, 0};
  for (int d = last - 1; d >= 0; --d) {
    const int64_t i = row % a.shape[d];
    row /= a.shape[d];
    ooff += i * a.ostr[d];
    for (int k = 0; k < a.n_in; ++k) ioff[k] += i * a.istr[k][d];
  }
  Tout *o = static_cast<Tout *>(a.out) + ooff;
#pragma unroll
  for (int u = 0; u < kRowsUnroll; ++u) {
    const int64_t c = (chunk * kRowsUnroll + u) * kRowsThreads + threadIdx.x;
    if (c < n) {
      float f[3] = {0.0f, 0.0f, 0.0f};
      for (int k = 0; k < a.n_in; ++k)
        f[k] = Elem<Tin>::load(static_cast<const Tin *>(a.in[k]) + ioff[k] + c * a.istr[k][last]);
      Elem<Tout>::store(o + c, ew_apply_rt<sizeof(Tout) == 2>(a.op, f[0], f[1], f[2], a.s0));
    }
  }
}

// family 3: one thread per element
template <typename Tin, typename Tout>
__global__ __launch_bounds__(256) void ew_general_kernel(StridedArgs a) {
  int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= a.total) return;
  int64_t ooff = 0, ioff[3] = {0, 0, 0};
  for (int d = a.nd - 1; d >= 0; --d) {
    const int64_t i = e % a.shape[d];
    e /= a.shape[d];
    ooff += i * a.ostr[d];
    for (int k = 0; k < a.n_in; ++k) ioff[k] += i * a.istr[k][d];
  }
  float f[3] = {0.0f, 0.0f, 0.0f};
  for (int k = 0; k < a.n_in; ++k) f[k] = Elem<Tin>::load(static_cast<const Tin *>(a.in[k]) + ioff[k]);
  Elem<Tout>::store(static_cast<Tout *>(a.out) + ooff, ew_apply_rt<sizeof(Tout) == 2>(a.op, f[0], f[1], f[2], a.s0));
}

// ------------------------------------------------------------------------------------------------
// family 2: 2-d, transposed inputs staged through LDS tiles
struct TransArgs {
  const void *in[3];
  void *out;
  int64_t rows, cols;
  int64_t ostr0;
  int64_t istr0[3], istr1[3];
  int transposed[3];
  int slot[3];   // vector form: which LDS tile a transposed input uses
  float s0;
};

constexpr int kTile = 64;

template <int OP, typename Tin, typename Tout, int NIN>
__global__ __launch_bounds__(256) void ew_transpose_kernel(TransArgs a, int64_t tiles_c) {
  __shared__ float tile[NIN][kTile][kTile + 1];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int64_t r0 = ((int64_t)blockIdx.x / tiles_c) * kTile;
  const int64_t c0 = ((int64_t)blockIdx.x % tiles_c) * kTile;
#pragma unroll
  for (int k = 0; k < NIN; ++k) {
    if (!a.transposed[k]) continue;
    const Tin *p = static_cast<const Tin *>(a.in[k]);
    const int64_t r = r0 + tx;  // this operand is contiguous along rows
#pragma unroll 4
    for (int j = 0; j < kTile / 4; ++j) {
      const int cl = ty + 4 * j;
      const int64_t c = c0 + cl;
      float v = 0.0f;
      if (r < a.rows && c < a.cols) v = Elem<Tin>::load(p + r * a.istr0[k] + c * a.istr1[k]);
      tile[k][cl][tx] = v;
    }
  }
  __syncthreads();
  const int64_t c = c0 + tx;
#pragma unroll 4
  for (int j = 0; j < kTile / 4; ++j) {
    const int rl = ty + 4 * j;
    const int64_t r = r0 + rl;
    if (r < a.rows && c < a.cols) {
      float f[3] = {0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int k = 0; k < NIN; ++k) {
        if (a.transposed[k]) f[k] = tile[k][tx][rl];
        else f[k] = Elem<Tin>::load(static_cast<const Tin *>(a.in[k]) + r * a.istr0[k] + c * a.istr1[k]);
      }
      Elem<Tout>::store(static_cast<Tout *>(a.out) + r * a.ostr0 + c, ew_apply<OP, sizeof(Tout) == 2>(f[0], f[1], f[2], a.s0));
    }
  }
}

// family 2, vector form: 16-byte global accesses on every operand.  A tile is TC (64 or 128) columns x
// 16 vectors of rows (64 fp32 / 128 bf16 rows).  A transposed input is read along its unit-stride (row) axis,
// 16 bytes per lane and 256 contiguous bytes per 16 lanes, and parked in LDS as [column][row], the
// 16-byte chunk index XORed with (column / E) so that both the 16-byte writes and the later
// element reads along a column are free of bank conflicts.  The compute phase then walks rows:
// each lane produces E consecutive columns of one row, gathering the transposed operands element by
// element from LDS and everything else with 16-byte global loads, and stores 16 bytes.
template <int OP, typename T, int NIN, int TC>
__global__ __launch_bounds__(256) void ew_transpose_vec_kernel(TransArgs a, int64_t tiles_c) {
  constexpr int E = 16 / (int)sizeof(T);
  constexpr int TR = 16 * E;
  constexpr int VPR = TC / E, RPP = 256 / VPR;
  extern __shared__ __align__(16) char tiles[];   // one tile of TC * 256 bytes per transposed input
  const int t = threadIdx.x;
  // Diagonal tile order: blocks that run at the same time differ in their row tile AND their column
  // tile.  With a power-of-two leading dimension, neighbours that differed in one of them only would
  // send all their strided 256-byte reads of one operand to the same few memory channels.
  const int64_t tiles_r = (a.rows + TR - 1) / TR;
  const int64_t ct = (int64_t)blockIdx.x % tiles_c;
  const int64_t rt = ((int64_t)blockIdx.x / tiles_c + ct) % tiles_r;
  const int64_t r0 = rt * TR, c0 = ct * TC;
  {
    const int rchunk = t & 15, cl = t >> 4;
    const int64_t r = r0 + rchunk * E;
#pragma unroll
    for (int k = 0; k < NIN; ++k) {
      if (!a.transposed[k]) continue;
      const T *p = static_cast<const T *>(a.in[k]);
#pragma unroll
      for (int j = 0; j < TC / 16; ++j) {
        const int c = cl + 16 * j;
        Vec16<T> v;
        v.raw = {};
        if (r < a.rows && c0 + c < a.cols) v.load_nt(p + r + (c0 + c) * a.istr1[k]);
        const int key = (c / E) & 15;
        *reinterpret_cast<decltype(v.raw) *>(tiles + a.slot[k] * (TC * 256) + c * 256 + ((rchunk ^ key) << 4)) = v.raw;
      }
    }
  }
  // The other operands' loads for all passes are issued now, next to the tile loads, so that every
  // global read of the block is in flight at once and only one memory latency is exposed.
  constexpr int NP = TR / RPP;
  const int cq = t % VPR, rr = t / VPR;
  const int64_t c = c0 + cq * E;
  Vec16<T> d[NIN][NP];
#pragma unroll
  for (int k = 0; k < NIN; ++k) {
    if (a.transposed[k]) continue;
    const T *p = static_cast<const T *>(a.in[k]);
#pragma unroll
    for (int pass = 0; pass < NP; ++pass) {
      const int64_t r = r0 + rr + pass * RPP;
      d[k][pass].raw = {};
      if (r < a.rows && c < a.cols) {
        if (a.istr1[k] == 0) {
          const float v = Elem<T>::load(p + r * a.istr0[k]);
#pragma unroll
          for (int i = 0; i < E; ++i) d[k][pass].set(i, v);
        } else if (a.istr0[k] == 0) d[k][pass].load(p + c);
        else d[k][pass].load_nt(p + r * a.istr0[k] + c);
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int pass = 0; pass < NP; ++pass) {
    const int rl = rr + pass * RPP;
    const int64_t r = r0 + rl;
    if (r < a.rows && c < a.cols) {
      float f[3][E];
#pragma unroll
      for (int k = 0; k < NIN; ++k) {
        if (a.transposed[k]) {
          const char *base = tiles + a.slot[k] * (TC * 256) + (((rl / E) ^ (cq & 15)) << 4) + (rl % E) * (int)sizeof(T);
#pragma unroll
          for (int i = 0; i < E; ++i) f[k][i] = Elem<T>::load(reinterpret_cast<const T *>(base + (cq * E + i) * 256));
        } else {
#pragma unroll
          for (int i = 0; i < E; ++i) f[k][i] = d[k][pass].get(i);
        }
      }
      Vec16<T> o;
#pragma unroll
      for (int i = 0; i < E; ++i)
        o.set(i, ew_apply<OP, sizeof(T) == 2>(f[0][i], NIN > 1 ? f[1][i] : 0.0f, NIN > 2 ? f[2][i] : 0.0f, a.s0));
      o.store_nt(static_cast<T *>(a.out) + r * a.ostr0 + c);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// dispatch
template <int OP, typename Tin, typename Tout>
chn_status launch_fast(const Plan &p, const chn_array *const *in, const chn_array *out, float s0, hipStream_t st) {
  constexpr int NIN = kArity[OP];
  if (p.family == 0) {
    FlatArgs a{};
    for (int k = 0; k < NIN; ++k) { a.in[k] = in[k]->data; a.mode[k] = p.mode[k]; a.period[k] = p.period[k]; }
    a.out = out->data; a.total = p.total; a.s0 = s0;
    constexpr int E = (sizeof(Tin) == 2 || sizeof(Tout) == 2) ? 8 : 4;
    int64_t nvec = p.total / E;
    int64_t blocks = (nvec + kFlatThreads * kFlatUnroll - 1) / (kFlatThreads * kFlatUnroll);
    if (blocks < 1) blocks = 1;
    if (blocks > 0x7fffffff) return fail(CHN_ERR_SHAPE, "elementwise: array too large");
    hipLaunchKernelGGL((ew_flat_kernel<OP, Tin, Tout, NIN>), dim3((unsigned)blocks), dim3(kFlatThreads), 0, st, a);
    return check_launch("elementwise flat");
  }
  // family 2
  TransArgs a{};
  a.out = out->data; a.rows = p.shape[0]; a.cols = p.shape[1]; a.ostr0 = p.ostr[0]; a.s0 = s0;
  for (int k = 0; k < NIN; ++k) {
    a.in[k] = in[k]->data; a.istr0[k] = p.istr[k][0]; a.istr1[k] = p.istr[k][1]; a.transposed[k] = p.transposed[k];
  }
  int64_t tr = (a.rows + kTile - 1) / kTile, tc = (a.cols + kTile - 1) / kTile;
  if (tr * tc > 0x7fffffff) return fail(CHN_ERR_SHAPE, "elementwise: array too large");
  if constexpr (NIN > 0) {
    if constexpr (std::is_same<Tin, Tout>::value) {
      if (p.tvec) {
        constexpr int TRV = 16 * (16 / (int)sizeof(Tin));
        const int64_t trv = (a.rows + TRV - 1) / TRV;
        if (trv * tc > 0x7fffffff) return fail(CHN_ERR_SHAPE, "elementwise: array too large");
        int nslots = 0;
        for (int k = 0; k < NIN; ++k) a.slot[k] = a.transposed[k] ? nslots++ : 0;
        // fp32: tiles of 128 columns where the LDS tiles fit (rows of the other operands and of the output
        // are then touched in 512-byte pieces: +4 % at 8192 x 8192; bf16 gains nothing from it)
        if (sizeof(Tin) == 4 && nslots * 128 * 256 <= 65536) {
          const int64_t tcw = (a.cols + 127) / 128;
          hipLaunchKernelGGL((ew_transpose_vec_kernel<OP, Tin, NIN, 128>), dim3((unsigned)(trv * tcw)), dim3(256), nslots * 128 * 256, st, a, tcw);
        } else {
          hipLaunchKernelGGL((ew_transpose_vec_kernel<OP, Tin, NIN, 64>), dim3((unsigned)(trv * tc)), dim3(256), nslots * 64 * 256, st, a, tc);
        }
        return check_launch("elementwise transpose (vector)");
      }
    }
    hipLaunchKernelGGL((ew_transpose_kernel<OP, Tin, Tout, NIN>), dim3((unsigned)(tr * tc)), dim3(256), 0, st, a, tc);
  }
  return check_launch("elementwise transpose");
}

template <typename Tin, typename Tout>
chn_status launch_dtype(int op, const Plan &p, const chn_array *const *in, const chn_array *out, float s0, hipStream_t st) {
  if (p.family == 0 || p.family == 2) {
    switch (op) {
#define CHN_CASE(OPC) case OPC: return launch_fast<OPC, Tin, Tout>(p, in, out, s0, st);
      CHN_CASE(CHN_OP_COPY) CHN_CASE(CHN_OP_ADD) CHN_CASE(CHN_OP_SUB) CHN_CASE(CHN_OP_MUL)
      CHN_CASE(CHN_OP_MAD) CHN_CASE(CHN_OP_MAD_RELU) CHN_CASE(CHN_OP_RELU) CHN_CASE(CHN_OP_RELU_BWD)
      CHN_CASE(CHN_OP_GELU) CHN_CASE(CHN_OP_GELU_BWD) CHN_CASE(CHN_OP_SCALE) CHN_CASE(CHN_OP_AXPY)
      CHN_CASE(CHN_OP_ADD_RELU) CHN_CASE(CHN_OP_ADD_GELU) CHN_CASE(CHN_OP_FILL)
      CHN_CASE(CHN_OP_SIGMOID) CHN_CASE(CHN_OP_TANH) CHN_CASE(CHN_OP_SQRT) CHN_CASE(CHN_OP_EXP) CHN_CASE(CHN_OP_GELU_BWD2)
#undef CHN_CASE
    }
    return fail(CHN_ERR_OP, "elementwise: unknown op %d", op);
  }
  StridedArgs a{};
  a.out = out->data; a.nd = p.nd; a.n_in = p.n_in; a.op = op; a.s0 = s0; a.total = p.total;
  for (int d = 0; d < p.nd; ++d) {
    a.shape[d] = p.shape[d]; a.ostr[d] = p.ostr[d];
    for (int k = 0; k < p.n_in; ++k) a.istr[k][d] = p.istr[k][d];
  }
  for (int k = 0; k < p.n_in; ++k) a.in[k] = in[k]->data;
  if (p.family == 1) {
    int64_t n = p.shape[p.nd - 1];
    int64_t rows = p.total / n;
    int64_t cpr = (n + kRowsThreads * kRowsUnroll - 1) / (kRowsThreads * kRowsUnroll);
    if (rows * cpr > 0x7fffffff) return fail(CHN_ERR_SHAPE, "elementwise: array too large");
    hipLaunchKernelGGL((ew_rows_kernel<Tin, Tout>), dim3((unsigned)(rows * cpr)), dim3(kRowsThreads), 0, st, a, cpr);
    return check_launch("elementwise rows");
  }
  int64_t blocks = (p.total + 255) / 256;
  if (blocks > 0x7fffffff) return fail(CHN_ERR_SHAPE, "elementwise: array too large");
  hipLaunchKernelGGL((ew_general_kernel<Tin, Tout>), dim3((unsigned)blocks), dim3(256), 0, st, a);
  return check_launch("elementwise general");
}

}  // namespace
}  // namespace chn

extern "C" {

int chn_elementwise_plan(int op, int n_in, const chn_array *const *in, const chn_array *out) {
  chn::Plan p;
  chn_status st = chn::make_plan(op, n_in, in, out, &p);
  if (st != CHN_OK) return st;
  return p.family;
}

chn_status chn_elementwise_broadcast(int op, int n_in, const chn_array *const *in,
                                     const chn_array *out, const float *scalars, int n_scalars,
                                     chn_stream stream) {
  using namespace chn;
  Plan p;
  CHN_TRY(make_plan(op, n_in, in, out, &p));
  if (n_scalars < kScalars[op] || (kScalars[op] > 0 && !scalars))
    return fail(CHN_ERR_OP, "elementwise: op %d needs %d scalar(s)", op, kScalars[op]);
  if (p.total == 0) return CHN_OK;
  const float s0 = kScalars[op] > 0 ? scalars[0] : 0.0f;
  const int tin = n_in > 0 ? in[0]->dtype : out->dtype;
  hipStream_t st = as_stream(stream);
  if (tin == CHN_F32 && out->dtype == CHN_F32) return launch_dtype<float, float>(op, p, in, out, s0, st);
  if (tin == CHN_BF16 && out->dtype == CHN_BF16) return launch_dtype<bf16_raw, bf16_raw>(op, p, in, out, s0, st);
  if (tin == CHN_F32 && out->dtype == CHN_BF16) return launch_dtype<float, bf16_raw>(op, p, in, out, s0, st);
  return launch_dtype<bf16_raw, float>(op, p, in, out, s0, st);
}

}  // extern "C"
