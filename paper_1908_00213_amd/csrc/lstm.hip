// chn_lstm_fwd / chn_lstm_bwd: the point-wise part of an LSTM step (textbook cell, gate order
// i, f, g, o).  The gate pre-activations come from GEMMs; these kernels fuse the bias add, the four
// activations and the cell/hidden update (forward) and the whole gate back-propagation (backward)
// into one pass each.  The backward works from retained outputs only (activated gates and c), as the
// paper's Section "Function-wise Local Memory Usage Reduction" describes for tanh-like operations.
// A call moves a few megabytes, so it is launch-latency bound; one thread per (batch, unit) pair with
// accesses coalesced along the hidden axis.
// Mixed precision: the arrays that feed matrix products -- h, the incoming dh and the outgoing dz --
// may be bfloat16 (rounded to nearest even on store); z, the gates and the cell state stay fp32.
#include "common.h"

namespace chn {
namespace {

struct LstmArgs {
  int64_t B, H;
  const float *z; int64_t z_pitch;
  const float *bias;
  const float *c_prev; int64_t cp_pitch;
  float *c; int64_t c_pitch;
  void *h; int64_t h_pitch;
  float *gates; int64_t g_pitch;
};

template <typename TH>
__global__ __launch_bounds__(256) void lstm_fwd_kernel(LstmArgs a) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= a.B * a.H) return;
  const int64_t b = e / a.H, j = e % a.H;
  const float *zr = a.z + b * a.z_pitch;
  float zi = zr[j], zf = zr[a.H + j], zg = zr[2 * a.H + j], zo = zr[3 * a.H + j];
  if (a.bias) { zi += a.bias[j]; zf += a.bias[a.H + j]; zg += a.bias[2 * a.H + j]; zo += a.bias[3 * a.H + j]; }
  const float i = sigmoid_f(zi), f = sigmoid_f(zf), g = tanhf(zg), o = sigmoid_f(zo);
  const float cn = f * a.c_prev[b * a.cp_pitch + j] + i * g;
  a.c[b * a.c_pitch + j] = cn;
  Elem<TH>::store(static_cast<TH *>(a.h) + b * a.h_pitch + j, o * tanhf(cn));
  if (a.gates) {
    float *gr = a.gates + b * a.g_pitch;
    gr[j] = i; gr[a.H + j] = f; gr[2 * a.H + j] = g; gr[3 * a.H + j] = o;
  }
}

struct LstmBwdArgs {
  int64_t B, H;
  const float *gates; int64_t g_pitch;
  const float *c_prev; int64_t cp_pitch;
  const float *c; int64_t c_pitch;
  const void *dh; int64_t dh_pitch;
  const float *dc_next; int64_t dcn_pitch;
  void *dz; int64_t dz_pitch;
  float *dc_prev; int64_t dcp_pitch;
};

template <typename TDH, typename TDZ>
__global__ __launch_bounds__(256) void lstm_bwd_kernel(LstmBwdArgs a) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= a.B * a.H) return;
  const int64_t b = e / a.H, j = e % a.H;
  const float *gr = a.gates + b * a.g_pitch;
  const float i = gr[j], f = gr[a.H + j], g = gr[2 * a.H + j], o = gr[3 * a.H + j];
  const float tc = tanhf(a.c[b * a.c_pitch + j]);
  const float dh = Elem<TDH>::load(static_cast<const TDH *>(a.dh) + b * a.dh_pitch + j);
  const float d_o = dh * tc;
  const float dc = (a.dc_next ? a.dc_next[b * a.dcn_pitch + j] : 0.0f) + dh * o * (1.0f - tc * tc);
  const float di = dc * g, dg = dc * i, df = dc * a.c_prev[b * a.cp_pitch + j];
  a.dc_prev[b * a.dcp_pitch + j] = dc * f;
  TDZ *dr = static_cast<TDZ *>(a.dz) + b * a.dz_pitch;
  Elem<TDZ>::store(dr + j, di * i * (1.0f - i));
  Elem<TDZ>::store(dr + a.H + j, df * f * (1.0f - f));
  Elem<TDZ>::store(dr + 2 * a.H + j, dg * (1.0f - g * g));
  Elem<TDZ>::store(dr + 3 * a.H + j, d_o * o * (1.0f - o));
}

chn_status mat(const chn_array *a, const char *name, bool out, int64_t B, int64_t cols, int64_t *pitch, bool bf16_ok = false) {
  CHN_TRY(validate(a, name, out));
  if (a->dtype != CHN_F32 && !(bf16_ok && a->dtype == CHN_BF16))
    return fail(CHN_ERR_DTYPE, "lstm: %s must be F32%s", name, bf16_ok ? " or BF16" : "");
  int64_t r, c;
  CHN_TRY(row_major_2d(a, name, &r, &c, pitch));
  if (r != B || c != cols) return fail(CHN_ERR_SHAPE, "lstm: %s must have shape (%lld,%lld)", name, (long long)B, (long long)cols);
  return CHN_OK;
}

}  // namespace
}  // namespace chn

extern "C" {

chn_status chn_lstm_fwd(const chn_array *z, const chn_array *bias, const chn_array *c_prev,
                        const chn_array *c, const chn_array *h, const chn_array *gates,
                        chn_stream stream) {
  using namespace chn;
  CHN_TRY(validate(c_prev, "c_prev", false));
  if (c_prev->ndim != 2) return fail(CHN_ERR_NDIM, "lstm: c_prev must be 2-d");
  LstmArgs a{};
  a.B = c_prev->shape[0]; a.H = c_prev->shape[1];
  CHN_TRY(mat(c_prev, "c_prev", false, a.B, a.H, &a.cp_pitch));
  CHN_TRY(mat(z, "z", false, a.B, 4 * a.H, &a.z_pitch));
  CHN_TRY(mat(c, "c", true, a.B, a.H, &a.c_pitch));
  CHN_TRY(mat(h, "h", true, a.B, a.H, &a.h_pitch, true));
  if (gates) CHN_TRY(mat(gates, "gates", true, a.B, 4 * a.H, &a.g_pitch));
  if (bias) {
    CHN_TRY(validate(bias, "bias", false));
    if (bias->dtype != CHN_F32) return fail(CHN_ERR_DTYPE, "lstm: bias must be F32");
    if (bias->ndim != 1 || bias->shape[0] != 4 * a.H || !is_contiguous(bias))
      return fail(CHN_ERR_SHAPE, "lstm: bias must be a contiguous (%lld,) array", (long long)(4 * a.H));
  }
  if (a.B * a.H == 0) return CHN_OK;
  a.z = static_cast<const float *>(z->data);
  a.bias = bias ? static_cast<const float *>(bias->data) : nullptr;
  a.c_prev = static_cast<const float *>(c_prev->data);
  a.c = static_cast<float *>(c->data);
  a.h = h->data;
  a.gates = gates ? static_cast<float *>(gates->data) : nullptr;
  const int64_t blocks = (a.B * a.H + 255) / 256;
  if (blocks > 0x7fffffff) return fail(CHN_ERR_SHAPE, "lstm: too large");
  if (h->dtype == CHN_BF16) hipLaunchKernelGGL(lstm_fwd_kernel<bf16_raw>, dim3((unsigned)blocks), dim3(256), 0, as_stream(stream), a);
  else hipLaunchKernelGGL(lstm_fwd_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, as_stream(stream), a);
  return check_launch("lstm_fwd");
}

chn_status chn_lstm_bwd(const chn_array *gates, const chn_array *c_prev, const chn_array *c,
                        const chn_array *dh, const chn_array *dc_next, const chn_array *dz,
                        const chn_array *dc_prev, chn_stream stream) {
  using namespace chn;
  CHN_TRY(validate(c, "c", false));
  if (c->ndim != 2) return fail(CHN_ERR_NDIM, "lstm: c must be 2-d");
  LstmBwdArgs a{};
  a.B = c->shape[0]; a.H = c->shape[1];
  CHN_TRY(mat(c, "c", false, a.B, a.H, &a.c_pitch));
  CHN_TRY(mat(gates, "gates", false, a.B, 4 * a.H, &a.g_pitch));
  CHN_TRY(mat(c_prev, "c_prev", false, a.B, a.H, &a.cp_pitch));
  CHN_TRY(mat(dh, "dh", false, a.B, a.H, &a.dh_pitch, true));
  if (dc_next) CHN_TRY(mat(dc_next, "dc_next", false, a.B, a.H, &a.dcn_pitch));
  CHN_TRY(mat(dz, "dz", true, a.B, 4 * a.H, &a.dz_pitch, true));
  CHN_TRY(mat(dc_prev, "dc_prev", true, a.B, a.H, &a.dcp_pitch));
  if (a.B * a.H == 0) return CHN_OK;
  a.gates = static_cast<const float *>(gates->data);
  a.c_prev = static_cast<const float *>(c_prev->data);
  a.c = static_cast<const float *>(c->data);
  a.dh = dh->data;
  a.dc_next = dc_next ? static_cast<const float *>(dc_next->data) : nullptr;
  a.dz = dz->data;
  a.dc_prev = static_cast<float *>(dc_prev->data);
  const int64_t blocks = (a.B * a.H + 255) / 256;
  if (blocks > 0x7fffffff) return fail(CHN_ERR_SHAPE, "lstm: too large");
  const dim3 grid((unsigned)blocks), block(256);
  const bool hb = dh->dtype == CHN_BF16, zb = dz->dtype == CHN_BF16;
  if (hb && zb) hipLaunchKernelGGL((lstm_bwd_kernel<bf16_raw, bf16_raw>), grid, block, 0, as_stream(stream), a);
  else if (hb) hipLaunchKernelGGL((lstm_bwd_kernel<bf16_raw, float>), grid, block, 0, as_stream(stream), a);
  else if (zb) hipLaunchKernelGGL((lstm_bwd_kernel<float, bf16_raw>), grid, block, 0, as_stream(stream), a);
  else hipLaunchKernelGGL((lstm_bwd_kernel<float, float>), grid, block, 0, as_stream(stream), a);
  return check_launch("lstm_bwd");
}

}  // extern "C"
