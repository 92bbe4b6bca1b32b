// Host-side pieces of the C ABI that launch nothing: descriptor validation, error strings, version.
#include "common.h"

namespace chn {

char *last_error_buffer() {
  static thread_local char buf[512] = {0};
  return buf;
}

chn_status validate(const chn_array *a, const char *name, bool is_output) {
  if (!a) return fail(CHN_ERR_NULL, "%s: descriptor is NULL", name);
  if (a->ndim < 0 || a->ndim > CHN_MAX_NDIM)
    return fail(CHN_ERR_NDIM, "%s: ndim %d outside 0..%d", name, a->ndim, CHN_MAX_NDIM);
  int isz = dtype_size(a->dtype);
  if (isz == 0) return fail(CHN_ERR_DTYPE, "%s: unknown dtype %d", name, a->dtype);
  int64_t n = 1;
  for (int d = 0; d < a->ndim; ++d) {
    if (a->shape[d] < 0) return fail(CHN_ERR_SHAPE, "%s: shape[%d] = %lld < 0", name, d, (long long)a->shape[d]);
    n *= a->shape[d];
  }
  for (int d = 0; d < a->ndim; ++d) {
    int64_t s = a->strides[d];
    if (a->shape[d] <= 1) continue;  // the stride of a length-0/1 dimension is never used
    if (s < 0) return fail(CHN_ERR_STRIDE, "%s: strides[%d] = %lld is negative", name, d, (long long)s);
    if (s % isz) return fail(CHN_ERR_STRIDE, "%s: strides[%d] = %lld is not a multiple of the item size %d", name, d, (long long)s, isz);
    if (is_output && s == 0 && n > 0)
      return fail(CHN_ERR_STRIDE, "%s: output has stride 0 along dimension %d of length %lld", name, d, (long long)a->shape[d]);
  }
  if (n > 0 && !a->data) return fail(CHN_ERR_NULL, "%s: data pointer is NULL", name);
  if (n > 0 && reinterpret_cast<uintptr_t>(a->data) % isz)
    return fail(CHN_ERR_STRIDE, "%s: data pointer is not aligned to the item size", name);
  return CHN_OK;
}

bool is_contiguous(const chn_array *a) {
  int64_t expect = dtype_size(a->dtype);
  for (int d = a->ndim - 1; d >= 0; --d) {
    if (a->shape[d] == 0) return true;
    if (a->shape[d] != 1 && a->strides[d] != expect) return false;
    expect *= a->shape[d];
  }
  return true;
}

chn_status row_major_2d(const chn_array *a, const char *name, int64_t *rows, int64_t *cols,
                        int64_t *pitch) {
  if (a->ndim != 2) return fail(CHN_ERR_NDIM, "%s: expected a 2-d array, got ndim %d", name, a->ndim);
  int isz = dtype_size(a->dtype);
  *rows = a->shape[0];
  *cols = a->shape[1];
  if (a->shape[1] > 1 && a->strides[1] != isz)
    return fail(CHN_ERR_STRIDE, "%s: last axis must have unit stride", name);
  int64_t p = a->shape[0] > 1 ? a->strides[0] / isz : a->shape[1];
  if (a->shape[0] > 1 && p < a->shape[1])
    return fail(CHN_ERR_STRIDE, "%s: row pitch %lld smaller than the row length %lld", name, (long long)p, (long long)a->shape[1]);
  *pitch = p;
  return CHN_OK;
}

}  // namespace chn

extern "C" {

const char *chn_status_string(chn_status s) {
  switch (s) {
    case CHN_OK: return "ok";
    case CHN_ERR_NULL: return "null pointer";
    case CHN_ERR_NDIM: return "bad number of dimensions";
    case CHN_ERR_DTYPE: return "unsupported dtype combination";
    case CHN_ERR_SHAPE: return "shape mismatch";
    case CHN_ERR_STRIDE: return "unsupported strides";
    case CHN_ERR_OP: return "unknown operation";
    case CHN_ERR_AXIS: return "axis out of range";
    case CHN_ERR_WORKSPACE: return "workspace missing or too small";
    case CHN_ERR_LAUNCH: return "kernel launch failed";
    case CHN_ERR_COMPILE: return "user kernel does not compile";
  }
  return "unknown status";
}

const char *chn_last_error(void) { return chn::last_error_buffer(); }

int chn_version(void) { return 100; }

}  // extern "C"
