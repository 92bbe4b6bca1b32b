// User-defined kernels (Section "Custom CUDA Kernels" of the paper, figure "Example of a
// user-defined kernel"): the caller gives parameter lists ("float32 x, T y") and C++ snippets; the
// library wraps them into a complete gfx950 kernel, compiles it at run time with hipRTC, keeps the
// code object in memory and on disk, and launches it over NumPy-broadcast operands.
//
// Two kinds, as in the paper: the element-wise kernel applies the snippet to every element; the
// reduction kernel folds mapped elements by a binary operator.  A type that is not a concrete
// dtype name is a type parameter: it is bound by the arrays of the call, and one kernel object
// serves every binding (one compiled specialisation each).
//
// Host only: parsing, code generation, the compile cache, stride bookkeeping and the launch.
// Generated device code follows the shapes of the hand-written kernels: 16 bytes per lane with
// non-temporal accesses and one vector per thread where operands are contiguous, one thread per
// element with a full index decomposition elsewhere; reductions in a fixed order (bit-reproducible).
#include <hip/hiprtc.h>
#include <sys/stat.h>
#include <unistd.h>

#include <algorithm>
#include <atomic>
#include <cctype>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "common.h"

namespace chn {
namespace {

constexpr int kMaxParams = 12;

struct Param {
  std::string type, name;
  int concrete;  // chn_dtype, or -1 for a type parameter
};

struct Loaded {
  hipModule_t mod = nullptr;
  hipFunction_t fn = nullptr, fn2 = nullptr;
};

}  // namespace
}  // namespace chn

struct chn_user_kernel {
  int kind = 0;  // 0 element-wise, 1 reduction
  std::vector<chn::Param> in, out;
  std::string name, preamble, operation;                    // element-wise
  std::string map_expr, reduce_expr, post_expr, identity;   // reduction
  std::map<std::string, std::vector<char>> binaries;        // specialisation key -> code object
  std::map<std::string, chn::Loaded> loaded;                // "device|key" -> module
  std::mutex mu;
};

namespace chn {
namespace {

// ---- process-wide configuration and counters -----------------------------------------------------
std::mutex g_mu;
std::string g_cache_dir;   // empty = default
std::string g_arch;        // empty = ask the current device
std::atomic<long long> g_compiles{0}, g_disk_hits{0}, g_memory_hits{0};

std::string cache_dir() {
  std::lock_guard<std::mutex> l(g_mu);
  if (!g_cache_dir.empty()) return g_cache_dir;
  if (const char *e = getenv("CHN_KERNEL_CACHE_DIR")) return e;
  const char *home = getenv("HOME");
  if (!home || !*home) return std::string();   // no home and no configured directory: no disk cache (never a shared /tmp)
  return std::string(home) + "/.cache/libchn/kernels";
}

chn_status target_arch(std::string *arch) {
  {
    std::lock_guard<std::mutex> l(g_mu);
    if (!g_arch.empty()) { *arch = g_arch; return CHN_OK; }
  }
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess)
    return fail(CHN_ERR_LAUNCH, "user kernel: no GPU to ask for its architecture (and none was configured)");
  *arch = prop.gcnArchName;
  return CHN_OK;
}

// (directories this creates are private to the user: cached code objects are executed)
void mkdirs(const std::string &path) {
  for (size_t i = 1; i <= path.size(); ++i)
    if (i == path.size() || path[i] == '/') mkdir(path.substr(0, i).c_str(), 0700);
}

// A cached code object is only trusted when it is a regular file that belongs to this user and that
// nobody else may write.
bool trusted_file(FILE *f) {
  struct stat st;
  if (fstat(fileno(f), &st) != 0) return false;
  return S_ISREG(st.st_mode) && st.st_uid == geteuid() && (st.st_mode & (S_IWGRP | S_IWOTH)) == 0;
}

// 128 bits of FNV-1a (two offset bases) as hex: the file name of a cached code object
std::string digest(const std::string &s) {
  uint64_t h[2] = {1469598103934665603ull, 0x9ae16a3b2f90404full};
  for (int k = 0; k < 2; ++k)
    for (unsigned char c : s) { h[k] ^= c + (k ? 0x5bu : 0u); h[k] *= 1099511628211ull; }
  char buf[40];
  snprintf(buf, sizeof buf, "%016llx%016llx", (unsigned long long)h[0], (unsigned long long)h[1]);
  return buf;
}

// ---- parameter lists ---------------------------------------------------------------------------------
bool is_ident(const std::string &s) {
  if (s.empty() || !(isalpha((unsigned char)s[0]) || s[0] == '_')) return false;
  for (char c : s) if (!(isalnum((unsigned char)c) || c == '_')) return false;
  return true;
}

int concrete_dtype(const std::string &t) {
  if (t == "float32") return CHN_F32;
  if (t == "bfloat16") return CHN_BF16;
  if (t == "int32") return CHN_I32;
  if (t == "int64") return CHN_I64;
  return -1;
}

chn_status parse_params(const char *text, const char *what, std::vector<Param> *out) {
  if (!text) return fail(CHN_ERR_NULL, "user kernel: %s is NULL", what);
  std::string s(text);
  size_t pos = 0;
  while (pos <= s.size()) {
    size_t comma = s.find(',', pos);
    if (comma == std::string::npos) comma = s.size();
    std::string item = s.substr(pos, comma - pos);
    pos = comma + 1;
    std::vector<std::string> tok;
    size_t i = 0;
    while (i < item.size()) {
      while (i < item.size() && isspace((unsigned char)item[i])) ++i;
      size_t j = i;
      while (j < item.size() && !isspace((unsigned char)item[j])) ++j;
      if (j > i) tok.push_back(item.substr(i, j - i));
      i = j;
    }
    if (tok.empty()) {
      if (s.find_first_not_of(" \t\n") == std::string::npos) break;  // an empty list
      return fail(CHN_ERR_OP, "user kernel: empty entry in %s \"%s\"", what, text);
    }
    if (tok.size() != 2 || !is_ident(tok[0]) || !is_ident(tok[1]))
      return fail(CHN_ERR_OP, "user kernel: %s entry \"%s\" is not \"<type> <name>\"", what, item.c_str());
    if (tok[1].rfind("chn_", 0) == 0 || tok[1] == "i")
      return fail(CHN_ERR_OP, "user kernel: parameter name \"%s\" is reserved", tok[1].c_str());
    if (tok[0] == "float16" || tok[0] == "float64" || tok[0] == "raw")
      return fail(CHN_ERR_DTYPE, "user kernel: type \"%s\" is not supported (float32, bfloat16, int32, int64 or a type parameter)", tok[0].c_str());
    out->push_back(Param{tok[0], tok[1], concrete_dtype(tok[0])});
  }
  if ((int)out->size() > kMaxParams) return fail(CHN_ERR_OP, "user kernel: more than %d parameters in %s", kMaxParams, what);
  return CHN_OK;
}

chn_status check_names(const chn_user_kernel &k) {
  std::vector<std::string> seen;
  for (const auto *list : {&k.in, &k.out})
    for (const Param &p : *list) {
      if (std::find(seen.begin(), seen.end(), p.name) != seen.end())
        return fail(CHN_ERR_OP, "user kernel: parameter name \"%s\" appears twice", p.name.c_str());
      if (k.kind == 1 && (p.name == "a" || p.name == "b"))
        return fail(CHN_ERR_OP, "user kernel: \"a\" and \"b\" name the operands of the reduction");
      seen.push_back(p.name);
    }
  if (!is_ident(k.name)) return fail(CHN_ERR_OP, "user kernel: \"%s\" is not a valid kernel name", k.name.c_str());
  if (k.out.empty()) return fail(CHN_ERR_OP, "user kernel: no output parameter");
  return CHN_OK;
}

// ---- type binding for one call -----------------------------------------------------------------------
struct Binding {
  std::vector<int> in_dtype, out_dtype;   // storage dtype of every parameter (scalars: declared type)
  std::vector<bool> in_scalar;
  std::map<std::string, int> generic;     // type parameter -> dtype
};

const char *storage_type(int dt) {
  switch (dt) {
    case CHN_F32: return "float";
    case CHN_BF16: return "chn_bf16";
    case CHN_I32: return "int";
    default: return "long long";
  }
}
const char *compute_type(int dt) {
  switch (dt) {
    case CHN_F32: case CHN_BF16: return "float";
    case CHN_I32: return "int";
    default: return "long long";
  }
}

chn_status bind_types(const chn_user_kernel &k, int n_in, const chn_array *const *in, int n_out,
                      const chn_array *const *out, Binding *b) {
  if (n_in != (int)k.in.size() || n_out != (int)k.out.size())
    return fail(CHN_ERR_OP, "%s: declared with %zu inputs and %zu outputs, called with %d and %d",
                k.name.c_str(), k.in.size(), k.out.size(), n_in, n_out);
  if ((n_in && !in) || !out) return fail(CHN_ERR_NULL, "%s: argument list is NULL", k.name.c_str());
  b->in_dtype.assign(n_in, -1);
  b->out_dtype.assign(n_out, -1);
  b->in_scalar.assign(n_in, false);
  auto bind = [&](const Param &p, const chn_array *a, int *slot) -> chn_status {
    CHN_TRY(validate(a, p.name.c_str(), false));
    if (p.concrete >= 0) {
      if (a->dtype != p.concrete)
        return fail(CHN_ERR_DTYPE, "%s: parameter %s is declared %s but the array has dtype %d",
                    k.name.c_str(), p.name.c_str(), p.type.c_str(), a->dtype);
    } else {
      auto it = b->generic.find(p.type);
      if (it == b->generic.end()) b->generic[p.type] = a->dtype;
      else if (it->second != a->dtype)
        return fail(CHN_ERR_DTYPE, "%s: type parameter %s is bound to dtype %d but %s has dtype %d",
                    k.name.c_str(), p.type.c_str(), it->second, p.name.c_str(), a->dtype);
    }
    *slot = a->dtype;
    return CHN_OK;
  };
  for (int i = 0; i < n_in; ++i)
    if (in[i]) CHN_TRY(bind(k.in[i], in[i], &b->in_dtype[i]));
  for (int i = 0; i < n_out; ++i) {
    if (!out[i]) return fail(CHN_ERR_NULL, "%s: output %s is NULL", k.name.c_str(), k.out[i].name.c_str());
    CHN_TRY(bind(k.out[i], out[i], &b->out_dtype[i]));
  }
  for (int i = 0; i < n_in; ++i) {
    if (in[i]) continue;
    b->in_scalar[i] = true;
    const Param &p = k.in[i];
    if (p.concrete >= 0) { b->in_dtype[i] = p.concrete; continue; }
    auto it = b->generic.find(p.type);
    if (it == b->generic.end())
      return fail(CHN_ERR_DTYPE, "%s: scalar %s has type parameter %s, which no array of the call binds",
                  k.name.c_str(), p.name.c_str(), p.type.c_str());
    b->in_dtype[i] = it->second;
  }
  return CHN_OK;
}

// ---- broadcast geometry -----------------------------------------------------------------------------
struct Dims {
  int nd = 0;
  int64_t shape[CHN_MAX_NDIM] = {0};
  std::vector<std::vector<int64_t>> str;   // [operand][dim], element strides
  int64_t total() const { int64_t n = 1; for (int d = 0; d < nd; ++d) n *= shape[d]; return n; }
};

// Element strides of `a` broadcast (right-aligned) to `shape`; size-1 dimensions repeat.
chn_status broadcast_strides(const char *kname, const Param &p, const chn_array *a, int nd, const int64_t *shape,
                             std::vector<int64_t> *str) {
  if (a->ndim > nd) return fail(CHN_ERR_SHAPE, "%s: %s has more dimensions than the output", kname, p.name.c_str());
  const int isz = dtype_size(a->dtype), shift = nd - a->ndim;
  str->assign(nd, 0);
  for (int d = 0; d < nd; ++d) {
    const int id = d - shift;
    if (id < 0 || a->shape[id] == 1) continue;
    if (a->shape[id] != shape[d])
      return fail(CHN_ERR_SHAPE, "%s: %s has length %lld along a dimension of length %lld", kname, p.name.c_str(),
                  (long long)a->shape[id], (long long)shape[d]);
    (*str)[d] = a->strides[id] / isz;
  }
  return CHN_OK;
}

// Drop length-1 dimensions and merge neighbours that are jointly contiguous in every operand.  The
// order of the remaining dimensions is kept, so the flat index stays the C-order index.
void collapse(Dims *g) {
  const int nop = (int)g->str.size();
  int m = 0;
  for (int d = 0; d < g->nd; ++d) {
    if (g->shape[d] == 1) continue;
    g->shape[m] = g->shape[d];
    for (int k = 0; k < nop; ++k) g->str[k][m] = g->str[k][d];
    ++m;
  }
  int w = 0;
  for (int d = 1; d < m; ++d) {
    bool ok = true;
    for (int k = 0; k < nop && ok; ++k) ok = g->str[k][w] == g->str[k][d] * g->shape[d];
    if (ok) {
      g->shape[w] *= g->shape[d];
      for (int k = 0; k < nop; ++k) g->str[k][w] = g->str[k][d];
    } else {
      ++w;
      g->shape[w] = g->shape[d];
      for (int k = 0; k < nop; ++k) g->str[k][w] = g->str[k][d];
    }
  }
  g->nd = m == 0 ? 0 : w + 1;
  for (int k = 0; k < nop; ++k) g->str[k].resize(g->nd);
}

// ---- generated source: common prelude ---------------------------------------------------------------
const char *kPrelude = R"SRC(
typedef unsigned short chn_bf16;
template <typename S> struct chn_io;
template <> struct chn_io<float> {
  typedef float C;
  static __device__ __forceinline__ C ld(const float *p) { return *p; }
  static __device__ __forceinline__ C up(float s) { return s; }
  static __device__ __forceinline__ float pk(C v) { return v; }
};
template <> struct chn_io<chn_bf16> {
  typedef float C;
  static __device__ __forceinline__ C up(chn_bf16 s) { return __uint_as_float((unsigned)s << 16); }
  static __device__ __forceinline__ C ld(const chn_bf16 *p) { return up(*p); }
  static __device__ __forceinline__ chn_bf16 pk(C v) {           // round to nearest even; NaN stays NaN
    unsigned u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (chn_bf16)((u >> 16) | 0x40u);
    return (chn_bf16)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
  }
};
template <> struct chn_io<int> {
  typedef int C;
  static __device__ __forceinline__ C ld(const int *p) { return *p; }
  static __device__ __forceinline__ C up(int s) { return s; }
  static __device__ __forceinline__ int pk(C v) { return v; }
};
template <> struct chn_io<long long> {
  typedef long long C;
  static __device__ __forceinline__ C ld(const long long *p) { return *p; }
  static __device__ __forceinline__ C up(long long s) { return s; }
  static __device__ __forceinline__ long long pk(C v) { return v; }
};
template <int BYTES> struct chn_raw;
template <> struct chn_raw<2> { typedef unsigned short T; };
template <> struct chn_raw<4> { typedef unsigned T; };
template <> struct chn_raw<8> { typedef unsigned T __attribute__((ext_vector_type(2))); };
template <> struct chn_raw<16> { typedef unsigned T __attribute__((ext_vector_type(4))); };
template <typename S, int E> struct chn_pack {       // E consecutive elements moved as one access
  typedef typename chn_raw<E * sizeof(S)>::T R;
  union { R raw; S e[E]; };
  __device__ __forceinline__ void load(const S *p) { raw = __builtin_nontemporal_load((const R *)p); }
  __device__ __forceinline__ void store(S *p) const { __builtin_nontemporal_store(raw, (R *)p); }
};
template <typename C> __device__ __forceinline__ C chn_scalar(unsigned long long bits) {
  return (C)__longlong_as_double((long long)bits);
}
)SRC";

struct Src {
  std::string s;
  Src &operator<<(const std::string &t) { s += t; return *this; }
  Src &operator<<(const char *t) { s += t; return *this; }
  Src &operator<<(long long v) { s += std::to_string(v); return *this; }
  Src &operator<<(int v) { s += std::to_string(v); return *this; }
};

std::string typedefs(const Binding &b) {
  std::string s;
  for (const auto &g : b.generic) s += "  typedef " + std::string(compute_type(g.second)) + " " + g.first + ";\n";
  return s;
}

// Slot layout shared by every generated kernel: 8-byte slots; arrays first (inputs that are arrays
// in declaration order, then outputs), then one slot per scalar input (a double), then geometry.
struct Slots {
  std::vector<unsigned long long> v;
  void ptr(const void *p) { v.push_back((unsigned long long)(uintptr_t)p); }
  void i64(int64_t x) { v.push_back((unsigned long long)x); }
  void f64(double x) { unsigned long long u; memcpy(&u, &x, 8); v.push_back(u); }
};

// ---- compile cache ------------------------------------------------------------------------------------
chn_status compile(const std::string &kname, const std::string &src, const std::string &arch, std::vector<char> *code) {
  hiprtcProgram prog;
  if (hiprtcCreateProgram(&prog, src.c_str(), (kname + ".hip").c_str(), 0, nullptr, nullptr) != HIPRTC_SUCCESS)
    return fail(CHN_ERR_COMPILE, "%s: hiprtcCreateProgram failed", kname.c_str());
  const std::string archopt = "--offload-arch=" + arch;
  // packed fp32 arithmetic is switched off for every kernel of this library, generated ones included
  const char *opts[] = {archopt.c_str(), "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"};
  hiprtcResult r = hiprtcCompileProgram(prog, 7, opts);
  if (r != HIPRTC_SUCCESS) {
    size_t n = 0;
    hiprtcGetProgramLogSize(prog, &n);
    std::string log(n + 1, '\0');
    if (n) hiprtcGetProgramLog(prog, &log[0]);
    hiprtcDestroyProgram(&prog);
    // the first error line is what the user needs; the buffer holds 512 bytes
    size_t e = log.find("error:");
    std::string shown = e == std::string::npos ? log : log.substr(e);
    return fail(CHN_ERR_COMPILE, "%s: the snippet does not compile: %.400s", kname.c_str(), shown.c_str());
  }
  size_t n = 0;
  hiprtcGetCodeSize(prog, &n);
  code->resize(n);
  hiprtcGetCode(prog, code->data());
  hiprtcDestroyProgram(&prog);
  ++g_compiles;
  return CHN_OK;
}

// Code object for (key, source): memory, then disk, then the compiler (and then both are filled).
chn_status binary_for(chn_user_kernel *k, const std::string &key, const std::string &src, const std::vector<char> **code) {
  auto it = k->binaries.find(key);
  if (it != k->binaries.end()) { ++g_memory_hits; *code = &it->second; return CHN_OK; }
  std::string arch;
  CHN_TRY(target_arch(&arch));
  int rtc_major = 0, rtc_minor = 0;
  hiprtcVersion(&rtc_major, &rtc_minor);
  const std::string dir = cache_dir();
  const std::string file = dir + "/" + digest(src + "|" + arch + "|" + std::to_string(rtc_major) + "." + std::to_string(rtc_minor) +
                                              "|" + std::to_string(chn_version())) + ".hsaco";
  std::vector<char> buf;
  FILE *cached = dir.empty() ? nullptr : fopen(file.c_str(), "rb");
  if (FILE *f = cached) {
    long n = 0;
    if (trusted_file(f)) {
      fseek(f, 0, SEEK_END);
      n = ftell(f);
      fseek(f, 0, SEEK_SET);
    }
    if (n > 0) { buf.resize(n); if (fread(buf.data(), 1, n, f) != (size_t)n) buf.clear(); }
    fclose(f);
    if (!buf.empty() && (buf.size() < 4 || memcmp(buf.data(), "\177ELF", 4) != 0)) buf.clear();   // not a code object
  }
  if (!buf.empty()) {
    ++g_disk_hits;
  } else {
    CHN_TRY(compile(k->name, src, arch, &buf));
    if (!dir.empty()) mkdirs(dir);
    const std::string tmp = file + ".tmp" + std::to_string((long long)getpid());
    if (FILE *f = dir.empty() ? nullptr : fopen(tmp.c_str(), "wb")) {      // a cache that cannot be written is not an error
      bool ok = fchmod(fileno(f), 0600) == 0;       // whatever the umask: writable by the owner alone
      ok = fwrite(buf.data(), 1, buf.size(), f) == buf.size() && ok;
      ok = fclose(f) == 0 && ok;
      if (!ok || rename(tmp.c_str(), file.c_str()) != 0) unlink(tmp.c_str());
    }
  }
  *code = &(k->binaries[key] = std::move(buf));
  return CHN_OK;
}

chn_status function_for(chn_user_kernel *k, const std::string &key, const std::string &src, bool second, Loaded *out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return fail(CHN_ERR_LAUNCH, "%s: no current device", k->name.c_str());
  const std::string lkey = std::to_string(dev) + "|" + key;
  auto it = k->loaded.find(lkey);
  if (it != k->loaded.end()) { ++g_memory_hits; *out = it->second; return CHN_OK; }
  const std::vector<char> *code = nullptr;
  CHN_TRY(binary_for(k, key, src, &code));
  Loaded l;
  hipError_t e = hipModuleLoadData(&l.mod, code->data());
  if (e != hipSuccess) return fail(CHN_ERR_LAUNCH, "%s: loading the code object failed: %s", k->name.c_str(), hipGetErrorString(e));
  e = hipModuleGetFunction(&l.fn, l.mod, k->name.c_str());
  if (e == hipSuccess && second) e = hipModuleGetFunction(&l.fn2, l.mod, (k->name + "_finish").c_str());
  if (e != hipSuccess) {
    (void)hipModuleUnload(l.mod);
    return fail(CHN_ERR_LAUNCH, "%s: kernel symbol not found in the code object: %s", k->name.c_str(), hipGetErrorString(e));
  }
  k->loaded[lkey] = l;
  *out = l;
  return CHN_OK;
}

chn_status launch(const chn_user_kernel *k, hipFunction_t fn, unsigned gx, unsigned gy, unsigned block, Slots &s, int n_slots,
                  chn_stream stream) {
  if ((int)s.v.size() != n_slots)
    return fail(CHN_ERR_LAUNCH, "%s: internal error, %zu argument slots packed for a kernel that takes %d", k->name.c_str(), s.v.size(), n_slots);
  size_t bytes = s.v.size() * 8;
  void *extra[] = {HIP_LAUNCH_PARAM_BUFFER_POINTER, s.v.data(), HIP_LAUNCH_PARAM_BUFFER_SIZE, &bytes, HIP_LAUNCH_PARAM_END};
  hipError_t e = hipModuleLaunchKernel(fn, gx, gy, 1, block, 1, 1, 0, as_stream(stream), nullptr, extra);
  if (e != hipSuccess) return fail(CHN_ERR_LAUNCH, "%s: launch failed: %s", k->name.c_str(), hipGetErrorString(e));
  return CHN_OK;
}

// ---- element-wise kernel --------------------------------------------------------------------------------
struct EwPlan {
  Binding b;
  Dims g;                      // operands: array inputs in order, then outputs
  std::vector<int> arr_of_in;  // input index -> operand index, -1 for scalars
  int n_arr = 0, n_sc = 0;
  bool flat = false, rows = false, idx32 = false;
  int E = 1;
  std::vector<bool> full;      // flat: operand is full-size (else a single repeated element)
                               // rows: operand advances along the inner dimension (else it repeats)
  int64_t total = 0;
  std::string key, src;
  int n_slots = 0;
};

// Argument list of the snippet function: inputs by value in their compute type, outputs by
// reference, then the flat C-order index `i` of the output element.
std::string op_signature(const chn_user_kernel &k, const Binding &b) {
  std::string s;
  for (size_t i = 0; i < k.in.size(); ++i)
    s += std::string("const ") + compute_type(b.in_dtype[i]) + " " + k.in[i].name + ", ";
  for (size_t i = 0; i < k.out.size(); ++i)
    s += std::string(compute_type(b.out_dtype[i])) + " &" + k.out[i].name + ", ";
  return s + "const long long i";
}

std::string ew_source(const chn_user_kernel &k, const EwPlan &p) {
  const Binding &b = p.b;
  const int n_in = (int)k.in.size(), n_out = (int)k.out.size();
  Src o;
  o << kPrelude << "struct chn_slots { unsigned long long v[" << p.n_slots << "]; };\n" << k.preamble << "\n";
  o << "__device__ __forceinline__ void chn_op(" << op_signature(k, b) << ") {\n" << typedefs(b) << "  " << k.operation << ";\n}\n";
  o << "extern \"C\" __global__ __launch_bounds__(256) void " << k.name << "(const chn_slots chn_s) {\n";
  // operand pointers and scalars
  for (int i = 0, a = 0, c = 0; i < n_in; ++i) {
    if (b.in_scalar[i]) {
      o << "  const " << compute_type(b.in_dtype[i]) << " chn_c" << i << " = chn_scalar<" << compute_type(b.in_dtype[i])
        << ">(chn_s.v[" << p.n_arr + c << "]);\n";
      ++c;
    } else {
      o << "  const " << storage_type(b.in_dtype[i]) << " *chn_p" << a << " = (const " << storage_type(b.in_dtype[i])
        << " *)chn_s.v[" << a << "];\n";
      ++a;
    }
  }
  const int first_out = p.n_arr - n_out;
  for (int j = 0; j < n_out; ++j)
    o << "  " << storage_type(b.out_dtype[j]) << " *chn_p" << first_out + j << " = (" << storage_type(b.out_dtype[j])
      << " *)chn_s.v[" << first_out + j << "];\n";
  const int geo = p.n_arr + p.n_sc;
  o << "  const long long chn_n = (long long)chn_s.v[" << geo << "];\n";
  // call of the snippet with per-element values named chn_x<i> / chn_y<j>
  auto call = [&](const std::string &index) {
    std::string s = "chn_op(";
    for (int i = 0; i < n_in; ++i) s += (b.in_scalar[i] ? "chn_c" : "chn_x") + std::to_string(i) + ", ";
    for (int j = 0; j < n_out; ++j) s += "chn_y" + std::to_string(j) + ", ";
    return s + index + ");";
  };
  if (p.flat) {
    const int E = p.E;
    // repeated single elements are read once
    for (int i = 0; i < n_in; ++i) {
      const int a = p.arr_of_in[i];
      if (a >= 0 && !p.full[a])
        o << "  const " << compute_type(b.in_dtype[i]) << " chn_x" << i << " = chn_io<" << storage_type(b.in_dtype[i]) << ">::ld(chn_p" << a << ");\n";
    }
    o << "  const long long chn_nvec = chn_n / " << E << ";\n"
      << "  const long long chn_v = (long long)blockIdx.x * 256 + threadIdx.x;\n"
      << "  if (chn_v < chn_nvec) {\n";
    for (int i = 0; i < n_in; ++i) {
      const int a = p.arr_of_in[i];
      if (a >= 0 && p.full[a])
        o << "    chn_pack<" << storage_type(b.in_dtype[i]) << ", " << E << "> chn_k" << a << "; chn_k" << a << ".load(chn_p" << a << " + chn_v * " << E << ");\n";
    }
    for (int j = 0; j < n_out; ++j)
      o << "    chn_pack<" << storage_type(b.out_dtype[j]) << ", " << E << "> chn_k" << first_out + j << ";\n";
    o << "#pragma unroll\n    for (int chn_j = 0; chn_j < " << E << "; ++chn_j) {\n";
    for (int i = 0; i < n_in; ++i) {
      const int a = p.arr_of_in[i];
      if (a >= 0 && p.full[a])
        o << "      const " << compute_type(b.in_dtype[i]) << " chn_x" << i << " = chn_io<" << storage_type(b.in_dtype[i]) << ">::up(chn_k" << a << ".e[chn_j]);\n";
    }
    for (int j = 0; j < n_out; ++j) o << "      " << compute_type(b.out_dtype[j]) << " chn_y" << j << " = 0;\n";
    o << "      " << call("chn_v * " + std::to_string(E) + " + chn_j") << "\n";
    for (int j = 0; j < n_out; ++j)
      o << "      chn_k" << first_out + j << ".e[chn_j] = chn_io<" << storage_type(b.out_dtype[j]) << ">::pk(chn_y" << j << ");\n";
    o << "    }\n";
    for (int j = 0; j < n_out; ++j) o << "    chn_k" << first_out + j << ".store(chn_p" << first_out + j << " + chn_v * " << E << ");\n";
    o << "  }\n"
      << "  const long long chn_t = chn_nvec * " << E << " + chn_v;     // the ragged tail, one element per thread\n"
      << "  if (chn_t < chn_n && chn_v < " << E << ") {\n";
    for (int i = 0; i < n_in; ++i) {
      const int a = p.arr_of_in[i];
      if (a >= 0 && p.full[a])
        o << "    const " << compute_type(b.in_dtype[i]) << " chn_x" << i << " = chn_io<" << storage_type(b.in_dtype[i]) << ">::ld(chn_p" << a << " + chn_t);\n";
    }
    for (int j = 0; j < n_out; ++j) o << "    " << compute_type(b.out_dtype[j]) << " chn_y" << j << " = 0;\n";
    o << "    " << call("chn_t") << "\n";
    for (int j = 0; j < n_out; ++j)
      o << "    chn_p" << first_out + j << "[chn_t] = chn_io<" << storage_type(b.out_dtype[j]) << ">::pk(chn_y" << j << ");\n";
    o << "  }\n}\n";
    return o.s;
  }
  if (p.rows) {
    // two dimensions, every operand with inner stride 1 or 0 and rows that start on vector
    // boundaries: one vector of the inner dimension per thread (a bias row, a column operand and
    // pitched views all land here)
    const int E = p.E;
    const char *IDX = p.idx32 ? "unsigned" : "long long";
    o << "  const long long chn_v = (long long)blockIdx.x * 256 + threadIdx.x;\n  if (chn_v >= chn_n / " << E << ") return;\n"
      << "  const " << IDX << " chn_cvn = (" << IDX << ")chn_s.v[" << geo + 1 << "];\n"
      << "  const " << IDX << " chn_row = (" << IDX << ")chn_v / chn_cvn;\n"
      << "  const long long chn_cv = (long long)((" << IDX << ")chn_v - chn_row * chn_cvn);\n";
    for (int a = 0; a < p.n_arr; ++a)
      o << "  const long long chn_o" << a << " = (long long)chn_row * (long long)chn_s.v[" << geo + 2 + a << "]"
        << (p.full[a] ? std::string(" + chn_cv * ") + std::to_string(E) : std::string("")) << ";\n";
    for (int i = 0; i < n_in; ++i) {
      const int a = p.arr_of_in[i];
      if (a < 0) continue;
      if (p.full[a])
        o << "  chn_pack<" << storage_type(b.in_dtype[i]) << ", " << E << "> chn_k" << a << "; chn_k" << a << ".load(chn_p" << a << " + chn_o" << a << ");\n";
      else
        o << "  const " << compute_type(b.in_dtype[i]) << " chn_x" << i << " = chn_io<" << storage_type(b.in_dtype[i]) << ">::ld(chn_p" << a << " + chn_o" << a << ");\n";
    }
    for (int j = 0; j < n_out; ++j)
      o << "  chn_pack<" << storage_type(b.out_dtype[j]) << ", " << E << "> chn_k" << first_out + j << ";\n";
    o << "#pragma unroll\n  for (int chn_j = 0; chn_j < " << E << "; ++chn_j) {\n";
    for (int i = 0; i < n_in; ++i) {
      const int a = p.arr_of_in[i];
      if (a >= 0 && p.full[a])
        o << "    const " << compute_type(b.in_dtype[i]) << " chn_x" << i << " = chn_io<" << storage_type(b.in_dtype[i]) << ">::up(chn_k" << a << ".e[chn_j]);\n";
    }
    for (int j = 0; j < n_out; ++j) o << "    " << compute_type(b.out_dtype[j]) << " chn_y" << j << " = 0;\n";
    o << "    " << call("chn_v * " + std::to_string(E) + " + chn_j") << "\n";
    for (int j = 0; j < n_out; ++j)
      o << "    chn_k" << first_out + j << ".e[chn_j] = chn_io<" << storage_type(b.out_dtype[j]) << ">::pk(chn_y" << j << ");\n";
    o << "  }\n";
    for (int j = 0; j < n_out; ++j) o << "  chn_k" << first_out + j << ".store(chn_p" << first_out + j << " + chn_o" << first_out + j << ");\n";
    o << "}\n";
    return o.s;
  }
  // general: one thread per element, full index decomposition (32-bit when the count allows)
  const int nd = p.g.nd;
  const char *IDX = p.idx32 ? "unsigned" : "long long";
  o << "  const long long chn_e = (long long)blockIdx.x * 256 + threadIdx.x;\n  if (chn_e >= chn_n) return;\n";
  for (int a = 0; a < p.n_arr; ++a) o << "  long long chn_o" << a << " = 0;\n";
  o << "  " << IDX << " chn_rem = (" << IDX << ")chn_e;\n";
  for (int d = nd - 1; d >= 0; --d) {
    o << "  {\n    const " << IDX << " chn_sh = (" << IDX << ")chn_s.v[" << geo + 1 + d << "];\n"
      << "    const " << IDX << " chn_q = chn_rem / chn_sh;\n    const long long chn_i = (long long)(chn_rem - chn_q * chn_sh);\n    chn_rem = chn_q;\n";
    for (int a = 0; a < p.n_arr; ++a)
      o << "    chn_o" << a << " += chn_i * (long long)chn_s.v[" << geo + 1 + nd + a * nd + d << "];\n";
    o << "  }\n";
  }
  for (int i = 0; i < n_in; ++i) {
    const int a = p.arr_of_in[i];
    if (a >= 0)
      o << "  const " << compute_type(b.in_dtype[i]) << " chn_x" << i << " = chn_io<" << storage_type(b.in_dtype[i]) << ">::ld(chn_p" << a << " + chn_o" << a << ");\n";
  }
  for (int j = 0; j < n_out; ++j) o << "  " << compute_type(b.out_dtype[j]) << " chn_y" << j << " = 0;\n";
  o << "  " << call("chn_e") << "\n";
  for (int j = 0; j < n_out; ++j)
    o << "  chn_p" << first_out + j << "[chn_o" << first_out + j << "] = chn_io<" << storage_type(b.out_dtype[j]) << ">::pk(chn_y" << j << ");\n";
  o << "}\n";
  return o.s;
}

std::string dtype_key(const Binding &b) {
  std::string s;
  for (size_t i = 0; i < b.in_dtype.size(); ++i) s += std::to_string(b.in_dtype[i]) + (b.in_scalar[i] ? "s" : "a");
  s += ">";
  for (int d : b.out_dtype) s += std::to_string(d);
  return s;
}

chn_status ew_plan(chn_user_kernel *k, int n_in, const chn_array *const *in, int n_out, const chn_array *const *out, EwPlan *p) {
  CHN_TRY(bind_types(*k, n_in, in, n_out, out, &p->b));
  const char *kn = k->name.c_str();
  const chn_array *o0 = out[0];
  for (int j = 0; j < n_out; ++j) {
    CHN_TRY(validate(out[j], k->out[j].name.c_str(), true));
    if (out[j]->ndim != o0->ndim) return fail(CHN_ERR_SHAPE, "%s: outputs differ in shape", kn);
    for (int d = 0; d < o0->ndim; ++d)
      if (out[j]->shape[d] != o0->shape[d]) return fail(CHN_ERR_SHAPE, "%s: outputs differ in shape", kn);
  }
  p->g.nd = o0->ndim;
  for (int d = 0; d < o0->ndim; ++d) p->g.shape[d] = o0->shape[d];
  p->arr_of_in.assign(n_in, -1);
  std::vector<const chn_array *> arrs;
  for (int i = 0; i < n_in; ++i) {
    if (!in[i]) { ++p->n_sc; continue; }
    p->arr_of_in[i] = (int)arrs.size();
    arrs.push_back(in[i]);
    p->g.str.emplace_back();
    CHN_TRY(broadcast_strides(kn, k->in[i], in[i], p->g.nd, p->g.shape, &p->g.str.back()));
  }
  for (int j = 0; j < n_out; ++j) {
    arrs.push_back(out[j]);
    p->g.str.emplace_back();
    CHN_TRY(broadcast_strides(kn, k->out[j], out[j], p->g.nd, p->g.shape, &p->g.str.back()));
  }
  p->n_arr = (int)arrs.size();
  p->total = p->g.total();
  if (p->total == 0) return CHN_OK;
  collapse(&p->g);
  // flat: one merged dimension in which every operand advances by 1 or stands still, and every
  // full-size operand is aligned for its vector access
  int max_isz = 1;
  for (const chn_array *a : arrs) max_isz = std::max(max_isz, dtype_size(a->dtype));
  p->E = 16 / max_isz;
  p->flat = p->g.nd <= 1;
  p->full.assign(p->n_arr, true);
  for (int a = 0; a < p->n_arr && p->flat; ++a) {
    const int64_t st = p->g.nd == 0 ? 0 : p->g.str[a][0];
    const bool is_out = a >= p->n_arr - n_out;
    if (st == 0 && !is_out) p->full[a] = false;
    else if (st != 1 && !(p->g.nd == 0)) p->flat = false;
    if (p->full[a] && reinterpret_cast<uintptr_t>(arrs[a]->data) % (p->E * dtype_size(arrs[a]->dtype))) p->flat = false;
  }
  p->idx32 = p->total < 0x7fffffffll;
  if (!p->flat && p->g.nd == 2 && p->g.shape[1] % p->E == 0) {
    p->rows = true;
    for (int a = 0; a < p->n_arr && p->rows; ++a) {
      const int64_t s0 = p->g.str[a][0], s1 = p->g.str[a][1];
      const bool is_out = a >= p->n_arr - n_out;
      p->full[a] = s1 == 1;
      if (s1 != 1 && (s1 != 0 || is_out)) p->rows = false;
      if (p->full[a] && (s0 % p->E || reinterpret_cast<uintptr_t>(arrs[a]->data) % (p->E * dtype_size(arrs[a]->dtype)))) p->rows = false;
    }
  }
  Src key;
  key << "ew|" << dtype_key(p->b) << "|";
  if (p->rows) {
    key << "rows" << p->E << (p->idx32 ? "|i32|" : "|i64|");
    for (int a = 0; a < p->n_arr; ++a) key << (p->full[a] ? "f" : "s");
    p->n_slots = p->n_arr + p->n_sc + 2 + p->n_arr;
  } else if (p->flat) {
    key << "flat" << p->E << "|";
    for (int a = 0; a < p->n_arr; ++a) key << (p->full[a] ? "f" : "s");
    p->n_slots = p->n_arr + p->n_sc + 1;
  } else {
    if (p->g.nd == 0) {   // a single element that did not qualify for the flat form
      p->g.nd = 1; p->g.shape[0] = 1;
      for (auto &s : p->g.str) s.assign(1, 0);
    }
    key << "nd" << p->g.nd << (p->idx32 ? "|i32" : "|i64");
    p->n_slots = p->n_arr + p->n_sc + 1 + p->g.nd * (1 + p->n_arr);
  }
  p->key = key.s;
  p->src = ew_source(*k, *p);
  return CHN_OK;
}

void ew_slots(const EwPlan &p, int n_in, const chn_array *const *in, int n_out, const chn_array *const *out, const double *scalars, Slots *s) {
  for (int i = 0; i < n_in; ++i) if (in[i]) s->ptr(in[i]->data);
  for (int j = 0; j < n_out; ++j) s->ptr(out[j]->data);
  for (int c = 0; c < p.n_sc; ++c) s->f64(scalars[c]);
  s->i64(p.total);
  if (p.rows) {
    s->i64(p.g.shape[1] / p.E);
    for (int a = 0; a < p.n_arr; ++a) s->i64(p.g.str[a][0]);
  } else if (!p.flat) {
    for (int d = 0; d < p.g.nd; ++d) s->i64(p.g.shape[d]);
    for (int a = 0; a < p.n_arr; ++a)
      for (int d = 0; d < p.g.nd; ++d) s->i64(p.g.str[a][d]);
  }
}

// ---- reduction kernel ----------------------------------------------------------------------------------
struct RdPlan {
  Binding b;
  Dims go, gr;                 // output dimensions / reduced dimensions; operands: array inputs, then outputs (go only)
  std::vector<int> arr_of_in;
  int n_arr_in = 0, n_sc = 0, n_out = 0;
  int64_t n_res = 0, R = 0;    // number of results, elements folded into each
  bool per_thread = false;     // one thread per result (the contiguous dimension is kept) vs one block per result
  bool idx32 = false;
  int E = 1;                   // elements per vector access (1: scalar accesses)
  bool finish_block = false;   // second pass: one block per result (few results, many slices)
  int64_t slices = 1, chunk = 0;
  std::string key, src;
  int n_slots = 0;
};

constexpr int kAxisAll = CHN_AXIS_ALL;

// Two mappings, each in a scalar and a vector form:
//   per block   one workgroup folds one result (or one slice of it); lanes stride along the reduced
//               range -- taken when the reduced dimension is the contiguous one (row sums, full sums);
//               vector form: 16 bytes per lane along that range;
//   per thread  one thread folds one result; neighbouring threads hold neighbouring results -- taken
//               when a kept dimension is the contiguous one (column sums); vector form: each thread
//               holds E neighbouring results and reads them with one 16-byte access per row, and 16
//               such threads (row lanes) share a group of results, each walking every 16th row of
//               the slice; they meet in LDS in lane order.
// A long reduced range is cut into slices (grid dimension y) whose partial values a second kernel
// folds in slice order.
std::string rd_source(const chn_user_kernel &k, const RdPlan &p) {
  const Binding &b = p.b;
  const int n_in = (int)k.in.size(), n_out = (int)k.out.size();
  const int E = p.E;
  const std::string RT = compute_type(b.out_dtype[0]);
  Src o;
  o << kPrelude << "struct chn_slots { unsigned long long v[" << p.n_slots << "]; };\ntypedef " << RT << " chn_R;\n" << k.preamble << "\n";
  std::string in_sig, in_args;
  for (int i = 0; i < n_in; ++i) {
    in_sig += std::string("const ") + compute_type(b.in_dtype[i]) + " " + k.in[i].name + ", ";
    in_args += (b.in_scalar[i] ? "chn_c" : "chn_x") + std::to_string(i) + ", ";
  }
  std::string sc_sig, sc_args;     // scalars are also visible to the final expression
  for (int i = 0; i < n_in; ++i)
    if (b.in_scalar[i]) {
      sc_sig += std::string(", const ") + compute_type(b.in_dtype[i]) + " " + k.in[i].name;
      sc_args += ", chn_c" + std::to_string(i);
    }
  std::string out_sig, out_args;
  for (int j = 0; j < n_out; ++j) {
    out_sig += std::string(", ") + compute_type(b.out_dtype[j]) + " &" + k.out[j].name;
    out_args += ", chn_y" + std::to_string(j);
  }
  o << "__device__ __forceinline__ chn_R chn_map(" << in_sig << "const long long i) {\n" << typedefs(b) << "  return (chn_R)(" << k.map_expr << ");\n}\n";
  o << "__device__ __forceinline__ chn_R chn_fold(const chn_R a, const chn_R b) {\n" << typedefs(b) << "  return (chn_R)(" << k.reduce_expr << ");\n}\n";
  o << "__device__ __forceinline__ void chn_post(const chn_R a" << out_sig << sc_sig << ") {\n" << typedefs(b) << "  " << k.post_expr << ";\n}\n";
  const int n_arr = p.n_arr_in + n_out;
  const int geo = n_arr + p.n_sc;        // n_res, R, slices, chunk, partials, then shapes and strides
  const int ndo = p.go.nd, ndr = p.gr.nd;
  const int so = geo + 5, sr = so + ndo * (1 + n_arr);   // out dims: shape + strides per operand; reduce dims: shape + strides per input
  const char *IDX = p.idx32 ? "unsigned" : "long long";
  auto decl = [&](Src &s) {
    for (int i = 0, a = 0, c = 0; i < n_in; ++i) {
      if (b.in_scalar[i]) {
        s << "  const " << compute_type(b.in_dtype[i]) << " chn_c" << i << " = chn_scalar<" << compute_type(b.in_dtype[i]) << ">(chn_s.v[" << n_arr + c << "]);\n";
        ++c;
      } else {
        s << "  const " << storage_type(b.in_dtype[i]) << " *chn_p" << a << " = (const " << storage_type(b.in_dtype[i]) << " *)chn_s.v[" << a << "];\n";
        ++a;
      }
    }
    for (int j = 0; j < n_out; ++j)
      s << "  " << storage_type(b.out_dtype[j]) << " *chn_p" << p.n_arr_in + j << " = (" << storage_type(b.out_dtype[j]) << " *)chn_s.v[" << p.n_arr_in + j << "];\n";
    s << "  const long long chn_nres = (long long)chn_s.v[" << geo << "];\n  const long long chn_R_len = (long long)chn_s.v[" << geo + 1 << "];\n"
      << "  const long long chn_slices = (long long)chn_s.v[" << geo + 2 << "];\n  const long long chn_chunk = (long long)chn_s.v[" << geo + 3 << "];\n"
      << "  chn_R *chn_part = (chn_R *)chn_s.v[" << geo + 4 << "];\n  (void)chn_R_len; (void)chn_chunk; (void)chn_slices; (void)chn_part;\n";
  };
  // offsets of result `chn_res` in every operand
  auto out_offsets = [&](Src &s, bool inputs) {
    for (int a = inputs ? 0 : p.n_arr_in; a < n_arr; ++a) s << "  long long chn_o" << a << " = 0;\n";
    s << "  {\n    " << IDX << " chn_rem = (" << IDX << ")chn_res;\n";
    for (int d = ndo - 1; d >= 0; --d) {
      s << "    {\n      const " << IDX << " chn_sh = (" << IDX << ")chn_s.v[" << so + d << "];\n      const " << IDX
        << " chn_q = chn_rem / chn_sh;\n      const long long chn_i = (long long)(chn_rem - chn_q * chn_sh);\n      chn_rem = chn_q;\n";
      for (int a = inputs ? 0 : p.n_arr_in; a < n_arr; ++a)
        s << "      chn_o" << a << " += chn_i * (long long)chn_s.v[" << so + ndo + a * ndo + d << "];\n";
      s << "    }\n";
    }
    s << "  }\n";
  };
  // offsets chn_q<a> of reduce index chn_r in every array input
  auto reduce_offsets = [&](Src &s, const std::string &ind) {
    if (ndr == 1) {
      for (int a = 0; a < p.n_arr_in; ++a) s << ind << "const long long chn_q" << a << " = chn_o" << a << " + chn_r * (long long)chn_s.v[" << sr + 1 + a << "];\n";
      return;
    }
    for (int a = 0; a < p.n_arr_in; ++a) s << ind << "long long chn_q" << a << " = chn_o" << a << ";\n";
    s << ind << IDX << " chn_rr = (" << IDX << ")chn_r;\n";
    for (int d = ndr - 1; d >= 0; --d) {
      s << ind << "{\n" << ind << "  const " << IDX << " chn_sh = (" << IDX << ")chn_s.v[" << sr + d << "];\n" << ind << "  const " << IDX
        << " chn_q = chn_rr / chn_sh;\n" << ind << "  const long long chn_i = (long long)(chn_rr - chn_q * chn_sh);\n" << ind << "  chn_rr = chn_q;\n";
      for (int a = 0; a < p.n_arr_in; ++a)
        s << ind << "  chn_q" << a << " += chn_i * (long long)chn_s.v[" << sr + ndr + a * ndr + d << "];\n";
      s << ind << "}\n";
    }
  };
  // one mapped element at reduce index chn_r folded into chn_acc (scalar accesses)
  auto fold_one = [&](Src &s, const std::string &ind) {
    s << ind << "{\n";
    reduce_offsets(s, ind + "  ");
    for (int i = 0; i < n_in; ++i) {
      const int a = p.arr_of_in[i];
      if (a >= 0)
        s << ind << "  const " << compute_type(b.in_dtype[i]) << " chn_x" << i << " = chn_io<" << storage_type(b.in_dtype[i]) << ">::ld(chn_p" << a << " + chn_q" << a << ");\n";
    }
    s << ind << "  chn_acc = chn_fold(chn_acc, chn_map(" << in_args << "chn_res * chn_R_len + chn_r));\n" << ind << "}\n";
  };
  // final expression and stores for the result whose folded value is `acc`, outputs at offset chn_o<a> + `shift`
  auto finish = [&](Src &s, const std::string &ind, const std::string &acc, const std::string &shift) {
    s << ind << "{\n";
    for (int j = 0; j < n_out; ++j) s << ind << "  " << compute_type(b.out_dtype[j]) << " chn_y" << j << " = 0;\n";
    s << ind << "  chn_post(" << acc << out_args << sc_args << ");\n";
    for (int j = 0; j < n_out; ++j)
      s << ind << "  chn_p" << p.n_arr_in + j << "[chn_o" << p.n_arr_in + j << shift << "] = chn_io<" << storage_type(b.out_dtype[j]) << ">::pk(chn_y" << j << ");\n";
    s << ind << "}\n";
  };
  const std::string tree =
      "  chn_sm[threadIdx.x] = chn_acc;\n  __syncthreads();\n"
      "  for (int chn_w = 128; chn_w > 0; chn_w >>= 1) {\n"
      "    if ((int)threadIdx.x < chn_w) chn_sm[threadIdx.x] = chn_fold(chn_sm[threadIdx.x], chn_sm[threadIdx.x + chn_w]);\n"
      "    __syncthreads();\n  }\n  if (threadIdx.x != 0) return;\n  chn_acc = chn_sm[0];\n";

  o << "extern \"C\" __global__ __launch_bounds__(256) void " << k.name << "(const chn_slots chn_s) {\n";
  decl(o);
  if (p.per_thread && E > 1) {
    // 16 groups of E neighbouring results x 16 row lanes: a lane walks every 16th element of the
    // slice, the lanes of a group meet in LDS in a fixed order
    o << "  const int chn_tx = threadIdx.x & 15, chn_ty = threadIdx.x >> 4;\n"
      << "  __shared__ chn_R chn_sm[16][16 * " << E << " + 1];\n"
      << "  long long chn_res = ((long long)blockIdx.x * 16 + chn_tx) * " << E << ";\n"
      << "  const bool chn_live = chn_res < chn_nres;\n  if (!chn_live) chn_res = 0;   // (stays in the barrier; reads and writes nothing)\n";
  } else if (p.per_thread) {
    o << "  const long long chn_res = ((long long)blockIdx.x * 256 + threadIdx.x) * " << E << ";\n  if (chn_res >= chn_nres) return;\n";
  } else {
    o << "  __shared__ chn_R chn_sm[256];\n  const long long chn_res = blockIdx.x;\n";
  }
  out_offsets(o, true);
  o << "  const long long chn_lo = (long long)blockIdx.y * chn_chunk;\n"
    << "  const long long chn_hi = chn_lo + chn_chunk < chn_R_len ? chn_lo + chn_chunk : chn_R_len;\n";
  if (p.per_thread && E > 1) {
    // E neighbouring results per thread: the last kept dimension is contiguous in every input
    o << "  chn_R chn_acc[" << E << "];\n#pragma unroll\n  for (int chn_j = 0; chn_j < " << E << "; ++chn_j) chn_acc[chn_j] = (chn_R)(" << k.identity << ");\n";
    o << "#pragma unroll 4\n  for (long long chn_r = chn_lo + chn_ty; chn_live && chn_r < chn_hi; chn_r += 16) {\n";
    reduce_offsets(o, "    ");
    for (int i = 0; i < n_in; ++i) {
      const int a = p.arr_of_in[i];
      if (a >= 0) o << "    chn_pack<" << storage_type(b.in_dtype[i]) << ", " << E << "> chn_k" << a << "; chn_k" << a << ".load(chn_p" << a << " + chn_q" << a << ");\n";
    }
    o << "#pragma unroll\n    for (int chn_j = 0; chn_j < " << E << "; ++chn_j) {\n";
    for (int i = 0; i < n_in; ++i) {
      const int a = p.arr_of_in[i];
      if (a >= 0) o << "      const " << compute_type(b.in_dtype[i]) << " chn_x" << i << " = chn_io<" << storage_type(b.in_dtype[i]) << ">::up(chn_k" << a << ".e[chn_j]);\n";
    }
    o << "      chn_acc[chn_j] = chn_fold(chn_acc[chn_j], chn_map(" << in_args << "(chn_res + chn_j) * chn_R_len + chn_r));\n    }\n  }\n";
    o << "#pragma unroll\n  for (int chn_j = 0; chn_j < " << E << "; ++chn_j) chn_sm[chn_ty][chn_tx * " << E << " + chn_j] = chn_acc[chn_j];\n"
      << "  __syncthreads();\n  if (chn_ty != 0 || !chn_live) return;\n"
      << "#pragma unroll\n  for (int chn_j = 0; chn_j < " << E << "; ++chn_j) {\n    chn_R chn_a = chn_sm[0][chn_tx * " << E << " + chn_j];\n"
      << "#pragma unroll\n    for (int chn_y = 1; chn_y < 16; ++chn_y) chn_a = chn_fold(chn_a, chn_sm[chn_y][chn_tx * " << E << " + chn_j]);\n"
      << "    chn_acc[chn_j] = chn_a;\n  }\n";
    o << "  if (chn_slices > 1) {\n#pragma unroll\n    for (int chn_j = 0; chn_j < " << E << "; ++chn_j) chn_part[(long long)blockIdx.y * chn_nres + chn_res + chn_j] = chn_acc[chn_j];\n    return;\n  }\n";
    o << "#pragma unroll\n  for (int chn_j = 0; chn_j < " << E << "; ++chn_j)\n";
    // the E results differ only in the last kept dimension: their outputs are one stride apart
    std::string body;
    {
      Src t;
      t << "  {\n";
      for (int j = 0; j < n_out; ++j) t << "    " << compute_type(b.out_dtype[j]) << " chn_y" << j << " = 0;\n";
      t << "    chn_post(chn_acc[chn_j]" << out_args << sc_args << ");\n";
      for (int j = 0; j < n_out; ++j)
        t << "    chn_p" << p.n_arr_in + j << "[chn_o" << p.n_arr_in + j << " + chn_j * (long long)chn_s.v[" << so + ndo + (p.n_arr_in + j) * ndo + (ndo - 1)
          << "]] = chn_io<" << storage_type(b.out_dtype[j]) << ">::pk(chn_y" << j << ");\n";
      t << "  }\n";
      body = t.s;
    }
    o << body << "}\n";
  } else {
    o << "  chn_R chn_acc = (chn_R)(" << k.identity << ");\n";
    if (p.per_thread) {
      o << "#pragma unroll 8\n  for (long long chn_r = chn_lo; chn_r < chn_hi; ++chn_r)\n";
      fold_one(o, "  ");
    } else if (E > 1) {
      // the reduced range is contiguous in every input: 16 bytes per lane, then a scalar tail
      o << "  const long long chn_nv = (chn_hi - chn_lo) / " << E << ";\n#pragma unroll 4\n"
        << "  for (long long chn_vi = threadIdx.x; chn_vi < chn_nv; chn_vi += 256) {\n    const long long chn_r0 = chn_lo + chn_vi * " << E << ";\n";
      for (int i = 0; i < n_in; ++i) {
        const int a = p.arr_of_in[i];
        if (a >= 0) o << "    chn_pack<" << storage_type(b.in_dtype[i]) << ", " << E << "> chn_k" << a << "; chn_k" << a << ".load(chn_p" << a << " + chn_o" << a << " + chn_r0);\n";
      }
      o << "#pragma unroll\n    for (int chn_j = 0; chn_j < " << E << "; ++chn_j) {\n";
      for (int i = 0; i < n_in; ++i) {
        const int a = p.arr_of_in[i];
        if (a >= 0) o << "      const " << compute_type(b.in_dtype[i]) << " chn_x" << i << " = chn_io<" << storage_type(b.in_dtype[i]) << ">::up(chn_k" << a << ".e[chn_j]);\n";
      }
      o << "      chn_acc = chn_fold(chn_acc, chn_map(" << in_args << "chn_res * chn_R_len + chn_r0 + chn_j));\n    }\n  }\n"
        << "  for (long long chn_r = chn_lo + chn_nv * " << E << " + threadIdx.x; chn_r < chn_hi; chn_r += 256)\n";
      fold_one(o, "  ");
    } else {
      o << "#pragma unroll 4\n  for (long long chn_r = chn_lo + threadIdx.x; chn_r < chn_hi; chn_r += 256)\n";
      fold_one(o, "  ");
    }
    if (!p.per_thread) o << tree;
    o << "  if (chn_slices > 1) {\n    chn_part[(long long)blockIdx.y * chn_nres + chn_res] = chn_acc;\n    return;\n  }\n";
    finish(o, "  ", "chn_acc", "");
    o << "}\n";
  }
  // second pass: fold the slices of every result in a fixed order, then the final expression
  o << "extern \"C\" __global__ __launch_bounds__(256) void " << k.name << "_finish(const chn_slots chn_s) {\n";
  decl(o);
  if (p.finish_block) {
    o << "  __shared__ chn_R chn_sm[256];\n  const long long chn_res = blockIdx.x;\n"
      << "  chn_R chn_acc = (chn_R)(" << k.identity << ");\n"
      << "  for (long long chn_sl = threadIdx.x; chn_sl < chn_slices; chn_sl += 256) chn_acc = chn_fold(chn_acc, chn_part[chn_sl * chn_nres + chn_res]);\n"
      << tree;
  } else {
    // 64 neighbouring results per block, four lanes of slices each, combined in a fixed order
    o << "  __shared__ chn_R chn_sm[256];\n  const int chn_lane = threadIdx.x & 63, chn_grp = threadIdx.x >> 6;\n"
      << "  const long long chn_res = (long long)blockIdx.x * 64 + chn_lane;\n"
      << "  chn_R chn_acc = (chn_R)(" << k.identity << ");\n"
      << "  if (chn_res < chn_nres) {\n#pragma unroll 8\n"
      << "    for (long long chn_sl = chn_grp; chn_sl < chn_slices; chn_sl += 4) chn_acc = chn_fold(chn_acc, chn_part[chn_sl * chn_nres + chn_res]);\n  }\n"
      << "  chn_sm[threadIdx.x] = chn_acc;\n  __syncthreads();\n  if (chn_grp != 0 || chn_res >= chn_nres) return;\n"
      << "  chn_acc = chn_fold(chn_fold(chn_fold(chn_sm[chn_lane], chn_sm[64 + chn_lane]), chn_sm[128 + chn_lane]), chn_sm[192 + chn_lane]);\n";
  }
  out_offsets(o, false);
  finish(o, "  ", "chn_acc", "");
  o << "}\n";
  return o.s;
}

chn_status rd_plan(chn_user_kernel *k, int n_in, const chn_array *const *in, int n_out, const chn_array *const *out, int axis,
                   int keepdims, RdPlan *p) {
  CHN_TRY(bind_types(*k, n_in, in, n_out, out, &p->b));
  const char *kn = k->name.c_str();
  p->n_out = n_out;
  // common input shape (NumPy broadcasting among the array inputs)
  int nd = 0;
  int64_t shape[CHN_MAX_NDIM];
  bool any = false;
  for (int i = 0; i < n_in; ++i) if (in[i]) { nd = std::max(nd, (int)in[i]->ndim); any = true; }
  if (!any) return fail(CHN_ERR_OP, "%s: a reduction needs at least one array input", kn);
  for (int d = 0; d < nd; ++d) shape[d] = 1;
  for (int i = 0; i < n_in; ++i) {
    if (!in[i]) continue;
    const int shift = nd - in[i]->ndim;
    for (int d = 0; d < in[i]->ndim; ++d) {
      const int64_t len = in[i]->shape[d];
      if (len == 1) continue;
      if (shape[shift + d] != 1 && shape[shift + d] != len)
        return fail(CHN_ERR_SHAPE, "%s: inputs do not broadcast against each other along dimension %d", kn, shift + d);
      shape[shift + d] = len;
    }
  }
  // which dimensions are folded: one axis, all of them, or the set bits of CHN_AXES(mask)
  bool red[CHN_MAX_NDIM] = {false};
  if (axis == kAxisAll) {
    for (int d = 0; d < nd; ++d) red[d] = true;
  } else if (axis >= CHN_AXES(0)) {
    const int mask = axis - CHN_AXES(0);
    if (mask == 0 || (mask >> nd) != 0) return fail(CHN_ERR_AXIS, "%s: axis set 0x%x out of range for %d dimensions", kn, mask, nd);
    for (int d = 0; d < nd; ++d) red[d] = (mask >> d) & 1;
  } else {
    int ax = axis < 0 ? axis + nd : axis;
    if (ax < 0 || ax >= nd) return fail(CHN_ERR_AXIS, "%s: axis %d out of range for %d dimensions", kn, axis, nd);
    red[ax] = true;
  }
  // expected output shape
  int ond = 0;
  int64_t oshape[CHN_MAX_NDIM];
  for (int d = 0; d < nd; ++d) {
    if (!red[d]) oshape[ond++] = shape[d];
    else if (keepdims) oshape[ond++] = 1;
  }
  for (int j = 0; j < n_out; ++j) {
    CHN_TRY(validate(out[j], k->out[j].name.c_str(), true));
    bool ok = out[j]->ndim == ond;
    for (int d = 0; d < ond && ok; ++d) ok = out[j]->shape[d] == oshape[d];
    if (!ok) return fail(CHN_ERR_SHAPE, "%s: output %s does not have the reduced shape", kn, k->out[j].name.c_str());
  }
  // split the dimensions into kept and reduced ones, with element strides per operand
  p->arr_of_in.assign(n_in, -1);
  std::vector<std::vector<int64_t>> istr;
  for (int i = 0; i < n_in; ++i) {
    if (!in[i]) { ++p->n_sc; continue; }
    p->arr_of_in[i] = p->n_arr_in++;
    istr.emplace_back();
    CHN_TRY(broadcast_strides(kn, k->in[i], in[i], nd, shape, &istr.back()));
  }
  p->go.str.assign(p->n_arr_in + n_out, {});
  p->gr.str.assign(p->n_arr_in, {});
  int od = 0;
  for (int d = 0; d < nd; ++d) {
    Dims &g = red[d] ? p->gr : p->go;
    g.shape[g.nd++] = shape[d];
    for (int a = 0; a < p->n_arr_in; ++a) g.str[a].push_back(istr[a][d]);
    if (!red[d]) {
      for (int j = 0; j < n_out; ++j) {
        const int isz = dtype_size(out[j]->dtype);
        p->go.str[p->n_arr_in + j].push_back(out[j]->shape[od] == 1 ? 0 : out[j]->strides[od] / isz);
      }
      ++od;
    } else if (keepdims) {
      ++od;
    }
  }
  p->n_res = p->go.total();
  p->R = p->gr.total();
  if (p->n_res == 0) return CHN_OK;
  // which dimension is the contiguous one of the first array input decides the mapping
  int64_t best_o = INT64_MAX, best_r = INT64_MAX;
  for (int d = 0; d < p->go.nd; ++d) if (p->go.shape[d] > 1 && p->go.str[0][d] > 0) best_o = std::min(best_o, p->go.str[0][d]);
  for (int d = 0; d < p->gr.nd; ++d) if (p->gr.shape[d] > 1 && p->gr.str[0][d] > 0) best_r = std::min(best_r, p->gr.str[0][d]);
  p->per_thread = best_o < best_r && p->n_res >= 64;
  collapse(&p->go);
  collapse(&p->gr);
  if (p->gr.nd == 0) { p->gr.nd = 1; p->gr.shape[0] = p->R; for (auto &s : p->gr.str) s.assign(1, 0); }
  p->idx32 = p->n_res < 0x7fffffffll && p->R < 0x7fffffffll;
  // vector accesses: 16 bytes per lane along the contiguous dimension when every array input
  // allows it (unit stride there, every other stride and the base address on vector boundaries)
  {
    int max_isz = 1;
    std::vector<const chn_array *> ins;
    for (int i = 0; i < n_in; ++i) if (in[i]) { ins.push_back(in[i]); max_isz = std::max(max_isz, dtype_size(in[i]->dtype)); }
    const int E = 16 / max_isz;
    bool ok = p->R > 0;
    for (int a = 0; a < p->n_arr_in && ok; ++a) {
      ok = reinterpret_cast<uintptr_t>(ins[a]->data) % (E * dtype_size(ins[a]->dtype)) == 0;
      if (p->per_thread) {
        const int last = p->go.nd - 1;
        ok = ok && last >= 0 && p->go.shape[last] % E == 0 && p->go.str[a][last] == 1;
        for (int d = 0; d < last && ok; ++d) ok = p->go.str[a][d] % E == 0;
        for (int d = 0; d < p->gr.nd && ok; ++d) ok = p->gr.str[a][d] % E == 0;
      } else {
        ok = ok && p->gr.nd == 1 && p->gr.str[a][0] == 1;
        for (int d = 0; d < p->go.nd && ok; ++d) ok = p->go.str[a][d] % E == 0;
      }
    }
    p->E = ok ? E : 1;
  }
  // slices of the reduced range so that the launch fills the chip; each slice at least 64 (per
  // thread) or 4096 (per block) elements long and a whole number of vectors
  const bool lanes = p->per_thread && p->E > 1;   // 16 result groups x 16 row lanes per block
  const int64_t blocks = lanes ? (p->n_res / p->E + 15) / 16 : p->per_thread ? (p->n_res / p->E + 255) / 256 : p->n_res;
  const int64_t min_len = p->per_thread ? 64 : 4096;
  int64_t s = blocks >= 2048 ? 1 : (2048 + blocks - 1) / blocks;
  s = std::min<int64_t>(s, std::max<int64_t>(1, p->R / min_len));
  if (lanes) {   // many short blocks stream best: 8 elements per lane (16 of 2-byte types), at most 16384 blocks
    s = std::max<int64_t>(1, p->R / (16 * (p->E > 4 ? 16 : 8)));
    if (blocks * s > 16384) s = std::max<int64_t>(1, 16384 / blocks);
  }
  s = std::min<int64_t>(s, 1024);
  p->chunk = p->R == 0 ? 1 : (p->R + s - 1) / s;
  p->chunk = (p->chunk + p->E - 1) / p->E * p->E;
  p->slices = p->R == 0 ? 1 : (p->R + p->chunk - 1) / p->chunk;
  p->finish_block = !p->per_thread && p->n_res <= 64;
  const int n_arr = p->n_arr_in + n_out;
  p->n_slots = n_arr + p->n_sc + 5 + p->go.nd * (1 + n_arr) + p->gr.nd * (1 + p->n_arr_in);
  Src key;
  key << "rd|" << dtype_key(p->b) << "|" << (p->per_thread ? "t" : "b") << p->E << (p->finish_block ? "B" : "T") << "|o" << p->go.nd << "r" << p->gr.nd
      << (p->idx32 ? "|i32" : "|i64");
  p->key = key.s;
  p->src = rd_source(*k, *p);
  return CHN_OK;
}

size_t rd_ws_bytes(const RdPlan &p) {
  if (p.n_res == 0 || p.slices <= 1) return 0;
  const size_t rsz = p.b.out_dtype[0] == CHN_I64 ? 8 : 4;
  return ((size_t)p.slices * p.n_res * rsz + 255) / 256 * 256;
}

void rd_slots(const RdPlan &p, int n_in, const chn_array *const *in, int n_out, const chn_array *const *out, const double *scalars,
              void *ws, Slots *s) {
  for (int i = 0; i < n_in; ++i) if (in[i]) s->ptr(in[i]->data);
  for (int j = 0; j < n_out; ++j) s->ptr(out[j]->data);
  for (int c = 0; c < p.n_sc; ++c) s->f64(scalars[c]);
  s->i64(p.n_res); s->i64(p.R); s->i64(p.slices); s->i64(p.chunk); s->ptr(ws);
  const int n_arr = p.n_arr_in + n_out;
  for (int d = 0; d < p.go.nd; ++d) s->i64(p.go.shape[d]);
  for (int a = 0; a < n_arr; ++a)
    for (int d = 0; d < p.go.nd; ++d) s->i64(p.go.str[a][d]);
  for (int d = 0; d < p.gr.nd; ++d) s->i64(p.gr.shape[d]);
  for (int a = 0; a < p.n_arr_in; ++a)
    for (int d = 0; d < p.gr.nd; ++d) s->i64(p.gr.str[a][d]);
}

chn_status need_scalars(const chn_user_kernel *k, int n_sc, const double *scalars) {
  if (n_sc > 0 && !scalars) return fail(CHN_ERR_NULL, "%s: the call has %d scalar parameters but `scalars` is NULL", k->name.c_str(), n_sc);
  return CHN_OK;
}

}  // namespace
}  // namespace chn

using namespace chn;

extern "C" {

chn_status chn_user_kernel_config(const char *cache_dir, const char *arch) {
  std::lock_guard<std::mutex> l(g_mu);
  if (cache_dir) g_cache_dir = cache_dir;     // "" = back to the default
  if (arch) g_arch = arch;                    // "" = back to asking the current device
  return CHN_OK;
}

void chn_user_kernel_stats(long long *compiles, long long *disk_hits, long long *memory_hits) {
  if (compiles) *compiles = g_compiles;
  if (disk_hits) *disk_hits = g_disk_hits;
  if (memory_hits) *memory_hits = g_memory_hits;
}

chn_status chn_elementwise_kernel_create(const char *in_params, const char *out_params, const char *operation,
                                         const char *name, const char *preamble, chn_user_kernel **out) {
  if (!out) return fail(CHN_ERR_NULL, "elementwise kernel: result pointer is NULL");
  *out = nullptr;
  if (!operation || !name) return fail(CHN_ERR_NULL, "elementwise kernel: operation or name is NULL");
  chn_user_kernel *k = new chn_user_kernel;
  k->kind = 0;
  k->name = name;
  k->operation = operation;
  k->preamble = preamble ? preamble : "";
  chn_status st = parse_params(in_params, "the input list", &k->in);
  if (st == CHN_OK) st = parse_params(out_params, "the output list", &k->out);
  if (st == CHN_OK) st = check_names(*k);
  if (st != CHN_OK) { delete k; return st; }
  *out = k;
  return CHN_OK;
}

chn_status chn_reduction_kernel_create(const char *in_params, const char *out_params, const char *map_expr,
                                       const char *reduce_expr, const char *post_map_expr, const char *identity,
                                       const char *name, const char *preamble, chn_user_kernel **out) {
  if (!out) return fail(CHN_ERR_NULL, "reduction kernel: result pointer is NULL");
  *out = nullptr;
  if (!map_expr || !reduce_expr || !post_map_expr || !identity || !name)
    return fail(CHN_ERR_NULL, "reduction kernel: an expression or the name is NULL");
  chn_user_kernel *k = new chn_user_kernel;
  k->kind = 1;
  k->name = name;
  k->map_expr = map_expr;
  k->reduce_expr = reduce_expr;
  k->post_expr = post_map_expr;
  k->identity = identity;
  k->preamble = preamble ? preamble : "";
  chn_status st = parse_params(in_params, "the input list", &k->in);
  if (st == CHN_OK) st = parse_params(out_params, "the output list", &k->out);
  if (st == CHN_OK) st = check_names(*k);
  if (st != CHN_OK) { delete k; return st; }
  *out = k;
  return CHN_OK;
}

void chn_user_kernel_destroy(chn_user_kernel *k) {
  if (!k) return;
  for (auto &l : k->loaded) (void)hipModuleUnload(l.second.mod);
  delete k;
}

chn_status chn_elementwise_kernel_prepare(chn_user_kernel *k, int n_in, const chn_array *const *in, int n_out,
                                          const chn_array *const *out) {
  if (!k || k->kind != 0) return fail(CHN_ERR_NULL, "elementwise kernel: not an element-wise kernel object");
  std::lock_guard<std::mutex> l(k->mu);
  EwPlan p;
  CHN_TRY(ew_plan(k, n_in, in, n_out, out, &p));
  if (p.total == 0) return CHN_OK;
  const std::vector<char> *code = nullptr;
  return binary_for(k, p.key, p.src, &code);
}

chn_status chn_elementwise_kernel_launch(chn_user_kernel *k, int n_in, const chn_array *const *in, int n_out,
                                         const chn_array *const *out, const double *scalars, chn_stream stream) {
  if (!k || k->kind != 0) return fail(CHN_ERR_NULL, "elementwise kernel: not an element-wise kernel object");
  std::lock_guard<std::mutex> l(k->mu);
  EwPlan p;
  CHN_TRY(ew_plan(k, n_in, in, n_out, out, &p));
  CHN_TRY(need_scalars(k, p.n_sc, scalars));
  if (p.total == 0) return CHN_OK;
  Loaded f;
  CHN_TRY(function_for(k, p.key, p.src, false, &f));
  Slots s;
  ew_slots(p, n_in, in, n_out, out, scalars, &s);
  const int64_t threads = p.rows ? p.total / p.E : p.flat ? std::max<int64_t>(p.total / p.E, p.E) : p.total;
  const int64_t blocks = (threads + 255) / 256;
  if (blocks > 0x7fffffffll) return fail(CHN_ERR_SHAPE, "%s: too many elements for one launch", k->name.c_str());
  return launch(k, f.fn, (unsigned)blocks, 1, 256, s, p.n_slots, stream);
}

size_t chn_reduction_kernel_workspace_bytes(chn_user_kernel *k, int n_in, const chn_array *const *in, int n_out,
                                            const chn_array *const *out, int axis, int keepdims) {
  if (!k || k->kind != 1) return 0;
  std::lock_guard<std::mutex> l(k->mu);
  RdPlan p;
  if (rd_plan(k, n_in, in, n_out, out, axis, keepdims, &p) != CHN_OK) return 0;
  return rd_ws_bytes(p);
}

chn_status chn_reduction_kernel_prepare(chn_user_kernel *k, int n_in, const chn_array *const *in, int n_out,
                                        const chn_array *const *out, int axis, int keepdims) {
  if (!k || k->kind != 1) return fail(CHN_ERR_NULL, "reduction kernel: not a reduction kernel object");
  std::lock_guard<std::mutex> l(k->mu);
  RdPlan p;
  CHN_TRY(rd_plan(k, n_in, in, n_out, out, axis, keepdims, &p));
  if (p.n_res == 0) return CHN_OK;
  const std::vector<char> *code = nullptr;
  return binary_for(k, p.key, p.src, &code);
}

chn_status chn_reduction_kernel_launch(chn_user_kernel *k, int n_in, const chn_array *const *in, int n_out,
                                       const chn_array *const *out, const double *scalars, int axis, int keepdims,
                                       void *ws, size_t ws_bytes, chn_stream stream) {
  if (!k || k->kind != 1) return fail(CHN_ERR_NULL, "reduction kernel: not a reduction kernel object");
  std::lock_guard<std::mutex> l(k->mu);
  RdPlan p;
  CHN_TRY(rd_plan(k, n_in, in, n_out, out, axis, keepdims, &p));
  CHN_TRY(need_scalars(k, p.n_sc, scalars));
  if (p.n_res == 0) return CHN_OK;
  CHN_TRY(check_ws(ws, ws_bytes, rd_ws_bytes(p), k->name.c_str()));
  Loaded f;
  CHN_TRY(function_for(k, p.key, p.src, true, &f));
  Slots s;
  rd_slots(p, n_in, in, n_out, out, scalars, p.slices > 1 ? ws : nullptr, &s);
  const int64_t gx = p.per_thread && p.E > 1 ? (p.n_res / p.E + 15) / 16 : p.per_thread ? (p.n_res / p.E + 255) / 256 : p.n_res;
  if (gx > 0x7fffffffll || p.slices > 65535) return fail(CHN_ERR_SHAPE, "%s: too many results for one launch", k->name.c_str());
  CHN_TRY(launch(k, f.fn, (unsigned)gx, (unsigned)p.slices, 256, s, p.n_slots, stream));
  if (p.slices > 1)
    CHN_TRY(launch(k, f.fn2, (unsigned)(p.finish_block ? p.n_res : (p.n_res + 63) / 64), 1, 256, s, p.n_slots, stream));
  return CHN_OK;
}

chn_status chn_user_kernel_source(chn_user_kernel *k, int n_in, const chn_array *const *in, int n_out,
                                  const chn_array *const *out, int axis, int keepdims, char *buf, size_t buf_bytes,
                                  size_t *needed) {
  if (!k) return fail(CHN_ERR_NULL, "user kernel: kernel object is NULL");
  std::lock_guard<std::mutex> l(k->mu);
  std::string src;
  if (k->kind == 0) {
    EwPlan p;
    CHN_TRY(ew_plan(k, n_in, in, n_out, out, &p));
    src = p.src;
  } else {
    RdPlan p;
    CHN_TRY(rd_plan(k, n_in, in, n_out, out, axis, keepdims, &p));
    src = p.src;
  }
  if (needed) *needed = src.size() + 1;
  if (buf && buf_bytes) {
    const size_t n = std::min(buf_bytes - 1, src.size());
    memcpy(buf, src.data(), n);
    buf[n] = '\0';
  }
  return CHN_OK;
}

}  // extern "C"
