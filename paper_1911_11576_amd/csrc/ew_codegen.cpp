// Kernel generation for all-elementwise fusion groups (paper Section 5.1: thread composition
// and kernel packing; Section 5.3: the stitched op is emitted as code).  The group's ops
// become one straight-line loop body over a chunk of consecutive elements: every parameter
// is loaded once, every intermediate is a register value, every output is stored once.
// Shapes, strides and constants are literals in the source, so index arithmetic for
// broadcast operands compiles to multiplications by constants.
//
// The source is compiled by the HIP run-time compiler for gfx950 (no GPU needed for that)
// and cached per process; loading the code object onto a device happens at the first launch.
#include "ew_ir.h"

#include <hip/hip_runtime.h>
#include <hip/hiprtc.h>
#include <unistd.h>

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <memory>
#include <mutex>

namespace fs {

namespace {

struct Emitter {
  std::string s;
  void line(const char* fmt, ...) __attribute__((format(printf, 2, 3))) {
    char buf[1024];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    s += buf;
    s += '\n';
  }
};

const char* kPreamble = R"SRC(
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
struct Args { const void* in[64]; void* out[16]; void* ws; };
#define UNROLL _Pragma("unroll")
static __device__ __forceinline__ float bits_f32(unsigned u) { return __builtin_bit_cast(float, u); }
static __device__ __forceinline__ unsigned f32_bits(float f) { return __builtin_bit_cast(unsigned, f); }
static __device__ __forceinline__ float bf16_lo(unsigned w) { return bits_f32(w << 16); }
static __device__ __forceinline__ float bf16_hi(unsigned w) { return bits_f32(w & 0xffff0000u); }
static __device__ __forceinline__ float f16_lo(unsigned w) { return (float)__builtin_bit_cast(_Float16, (unsigned short)(w & 0xffffu)); }
static __device__ __forceinline__ float f16_hi(unsigned w) { return (float)__builtin_bit_cast(_Float16, (unsigned short)(w >> 16)); }
// round to nearest even, NaN stays NaN: the hardware conversion (v_cvt_pk_bf16_f32, two values
// per instruction where the caller packs a pair)
static __device__ __forceinline__ unsigned to_bf16(float f) { return __builtin_bit_cast(unsigned short, (__bf16)f); }
static __device__ __forceinline__ unsigned to_f16(float f) { return __builtin_bit_cast(unsigned short, (_Float16)f); }
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
static __device__ __forceinline__ unsigned pack_to_bf16(float lo, float hi) { return __builtin_bit_cast(unsigned, __builtin_convertvector(f32x2{lo, hi}, bf16x2)); }
static __device__ __forceinline__ unsigned pack_to_f16(float lo, float hi) { return __builtin_bit_cast(unsigned, __builtin_convertvector(f32x2{lo, hi}, f16x2)); }
// e^x as one multiply and the hardware exp2 (groups with 16-bit tensors: the product's rounding costs |x| * 6e-8
// of relative accuracy, far inside their tolerance; expf's range fix-ups cost ten more instructions per value)
static __device__ __forceinline__ float exp_fast(float x) { return __builtin_amdgcn_exp2f(x * 1.4426950408889634f); }
// tanh(x) = 1 - 2 / (1 + e^(2x)) on the hardware exp2 and reciprocal: absolute error of a
// few 1e-7; exp2 overflow gives rcp(inf) = 0 -> 1, underflow gives 1 - 2 = -1
static __device__ __forceinline__ float tanh_fast(float x) {
  const float e = __builtin_amdgcn_exp2f(x * 2.885390081777927f);
  return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + e);
}
// tanh for fp32 groups, relative error below 1e-6 everywhere: the odd series up to x^9 below 0.3
// (next term 0.0089 x^11), 1 - 2 / (1 + e^(2|x|)) with the sign put back above (no cancellation there)
static __device__ __forceinline__ float tanh_f32(float x) {
  const float ax = __builtin_fabsf(x), x2 = x * x;
  const float p = x * (1.0f + x2 * (-0.33333334f + x2 * (0.13333334f + x2 * (-0.053968254f + x2 * 0.021869488f))));
  const float e = __builtin_amdgcn_exp2f(ax * 2.885390081777927f);
  const float t = 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + e);
  return ax < 0.3f ? p : __builtin_copysignf(t, x);
}
// erf for groups stored in 16 bits: 1 - (a1 t + ... + a5 t^5) e^(-x^2) with t = 1 / (1 + p |x|), the sign put
// back (the classical five-term rational form, absolute error 1.5e-7): one reciprocal, one exp2
static __device__ __forceinline__ float erf_fast(float x) {
  const float ax = __builtin_fabsf(x);
  const float t = __builtin_amdgcn_rcpf(1.0f + 0.3275911f * ax);
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  const float e = __builtin_amdgcn_exp2f(ax * ax * -1.4426950408889634f);
  return __builtin_copysignf(1.0f - poly * e, x);
}
// 1 / (1 + e^-x): exp2 overflow (x very negative) gives rcp(inf) = 0
static __device__ __forceinline__ float logistic(float x) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(x * -1.4426950408889634f));
}
// mul*h / (1 + exp2(h*(a0 + a1*h*h))), the tanh-form GELU; exp2 overflow gives rcp(inf) = 0
static __device__ __forceinline__ float gelu_tanh(float h, float mul, float a0, float a1) {
  const float e = __builtin_amdgcn_exp2f(h * (a0 + a1 * (h * h)));
  return (mul == 1.0f ? h : mul * h) * __builtin_amdgcn_rcpf(1.0f + e);
}
static __device__ __forceinline__ float round_bf16(float f) { return (float)(__bf16)f; }
static __device__ __forceinline__ float round_f16(float f) { return (float)(_Float16)f; }
)SRC";


std::string operand_text(const EwIrOperand& o) {
  char buf[64];
  if (o.kind == EW_FROM_NODE) snprintf(buf, sizeof buf, "t%d[j]", o.index);
  else if (o.kind == EW_FROM_VIEW) snprintf(buf, sizeof buf, "v%d[j]", o.index);
  else {
    uint32_t u;
    memcpy(&u, &o.cval, 4);
    snprintf(buf, sizeof buf, "bits_f32(0x%08xu)", u);
  }
  return buf;
}

std::string op_text(const EwIrNode& n, bool fast) {
  const std::string a = operand_text(n.opnd[0]);
  const std::string b = n.n_operands == 2 ? operand_text(n.opnd[1]) : std::string();
  switch (n.op) {
    case FS_ADD: return a + " + " + b;
    case FS_SUBTRACT: return a + " - " + b;
    case FS_MULTIPLY: return a + " * " + b;
    case FS_DIVIDE: return a + " / " + b;
    case FS_MAXIMUM: return "fmaxf(" + a + ", " + b + ")";
    case FS_NEGATE: return "-" + a;
    case FS_EXP: return (fast ? "exp_fast(" : "expf(") + a + ")";
    case FS_LOG: return "logf(" + a + ")";
    case FS_TANH: return (fast ? "tanh_fast(" : "tanh_f32(") + a + ")";
    case FS_RSQRT: return "rsqrtf(" + a + ")";
    case FS_SQRT: return "sqrtf(" + a + ")";
    case FS_ERF: return (fast ? "erf_fast(" : "erff(") + a + ")";
    case FS_LOGISTIC: return "logistic(" + a + ")";
    case EW_OP_ROUND_F16: return "round_f16(" + a + ")";
    case EW_OP_ROUND_BF16: return "round_bf16(" + a + ")";
    case EW_OP_GELU_TANH: {
      std::string t = "gelu_tanh(" + a;
      for (int q = 0; q < 3; ++q) {
        EwIrOperand c;
        c.kind = EW_FROM_CONST;
        c.cval = n.gelu[q];
        t += ", " + operand_text(c);
      }
      return t + ")";
    }
    case FS_CAUSAL_MASK: {
      // kept where the last index does not exceed the second-to-last one
      EwIrOperand fill;
      fill.kind = EW_FROM_CONST;
      fill.cval = n.opnd[1].cval;
      return "(i3 + j <= i2) ? " + a + " : " + operand_text(fill);
    }
    default: return a;
  }
}

}  // namespace

const char* ew_preamble() { return kPreamble; }

// Chunk width of a group: as many consecutive elements as one 16-byte access of the narrowest
// tensor holds, provided every row start stays aligned; otherwise one element.
static int chunk_width(const EwIr& ir) {
  const int64_t last = ir.shape[FS_MAX_RANK - 1];
  bool any32 = false;
  for (const EwIrView& v : ir.views) if (v.full && v.dtype == FS_F32) any32 = true;
  for (const EwIrNode& n : ir.nodes) if (n.out_ordinal >= 0 && n.out_dtype == FS_F32) any32 = true;
  auto fits = [&](int w) {
    if (last % w) return false;
    for (const EwIrView& v : ir.views) {
      if (v.full) continue;
      const int64_t ls = v.stride[FS_MAX_RANK - 1];
      if (ls != 0 && ls != 1) return false;
      if (ls == 1) for (int d = 0; d + 1 < FS_MAX_RANK; ++d) if (v.stride[d] % w) return false;
    }
    return true;
  };
  if (!any32 && fits(8)) return 8;
  if (fits(4)) return 4;
  return 1;
}

// The loop of one group over its chunks.  `blk` / `nblk` are the expressions for this group's
// workgroup index and workgroup count (the whole grid, or its share of a packed launch);
// `view_base` is where its operand views start in Args::in.
static void emit_part(Emitter& e, const EwIr& ir, int W, const std::string& blk, const std::string& nblk, int view_base) {
  bool need_idx = false;
  for (const EwIrView& v : ir.views) if (!v.full) need_idx = true;
  for (const EwIrNode& n : ir.nodes) if (n.op == FS_CAUSAL_MASK) need_idx = true;
  // A group that stores 16-bit values is compared at 16-bit accuracy: its tanh may take the
  // short hardware form.  fp32 groups keep the library function.
  bool fast = false;
  for (const EwIrView& v : ir.views) if (v.dtype != FS_F32) fast = true;
  for (const EwIrNode& n : ir.nodes) if (n.out_ordinal >= 0 && n.out_dtype != FS_F32) fast = true;

  e.line("  constexpr int W = %d;", W);
  e.line("  const long long nchunk = %lldll;", (long long)(ir.n / W));
  e.line("  for (long long ci = %s * blockDim.x + threadIdx.x; ci < nchunk; ci += %s * blockDim.x) {", blk.c_str(), nblk.c_str());
  e.line("    const long long e0 = ci * W;");
  if (need_idx) {
    // coordinates of the chunk's first element (the chunk never crosses a row: W divides the last extent)
    const bool small = ir.n <= 0x7fffffffLL;
    e.line("    %s r = (%s)e0;", small ? "unsigned" : "unsigned long long", small ? "unsigned" : "unsigned long long");
    for (int d = FS_MAX_RANK - 1; d >= 0; --d) {
      if (ir.shape[d] == 1) { e.line("    const long long i%d = 0;", d); continue; }
      const char* sfx = small ? "u" : "ull";
      e.line("    const long long i%d = r %% %lld%s; r /= %lld%s;", d, (long long)ir.shape[d], sfx, (long long)ir.shape[d], sfx);
    }
  }
  // ---- loads: every view once
  for (size_t k = 0; k < ir.views.size(); ++k) {
    const EwIrView& v = ir.views[k];
    const char* ty = v.dtype == FS_F32 ? "float" : "unsigned short";
    e.line("    float v%zu[W];", k);
    std::string off = "e0";
    bool splat = false;
    if (!v.full) {
      off.clear();
      for (int d = 0; d < FS_MAX_RANK; ++d) {
        if (v.stride[d] == 0) continue;
        char buf[64];
        snprintf(buf, sizeof buf, "%si%d * %lldll", off.empty() ? "" : " + ", d, (long long)v.stride[d]);
        off += buf;
      }
      if (off.empty()) off = "0";
      splat = v.stride[FS_MAX_RANK - 1] == 0;
    }
    e.line("    {");
    e.line("      const %s* p = static_cast<const %s*>(a.in[%zu]) + (%s);", ty, ty, view_base + k, off.c_str());
    // operands of the group's own shape stream through once; broadcast operands are re-read by
    // many threads and stay cached
    const char* ld = v.full ? "__builtin_nontemporal_load" : "*";
    if (splat || W == 1) {
      const char* conv = v.dtype == FS_F32 ? "p[0]" : v.dtype == FS_F16 ? "f16_lo(p[0])" : "bf16_lo(p[0])";
      e.line("      const float x = %s;", conv);
      e.line("      UNROLL for (int j = 0; j < W; ++j) v%zu[j] = x;", k);
    } else if (v.dtype == FS_F32) {
      for (int q = 0; q < W / 4; ++q) {
        e.line("      { const f32x4 x = %s(reinterpret_cast<const f32x4*>(p) + %d);", ld, q);
        e.line("        UNROLL for (int j = 0; j < 4; ++j) v%zu[%d + j] = x[j]; }", k, 4 * q);
      }
    } else {
      const char* lo = v.dtype == FS_F16 ? "f16_lo" : "bf16_lo";
      const char* hi = v.dtype == FS_F16 ? "f16_hi" : "bf16_hi";
      if (W == 8) e.line("      const u32x4 x = %s(reinterpret_cast<const u32x4*>(p));", ld);
      else e.line("      const u32x2 x = %s(reinterpret_cast<const u32x2*>(p));", ld);
      e.line("      UNROLL for (int j = 0; j < W / 2; ++j) { v%zu[2 * j] = %s(x[j]); v%zu[2 * j + 1] = %s(x[j]); }", k, lo, k, hi);
    }
    e.line("    }");
  }
  // ---- the ops, in order; outputs stored as soon as they exist
  for (const EwIrNode& n : ir.nodes) {
    e.line("    float t%d[W];", n.id);
    e.line("    UNROLL for (int j = 0; j < W; ++j) t%d[j] = %s;", n.id, op_text(n, fast).c_str());
    if (n.out_ordinal < 0) continue;
    e.line("    {");
    if (n.out_dtype == FS_F32) {
      e.line("      float* p = static_cast<float*>(a.out[%d]) + e0;", n.out_ordinal);
      if (W == 1) e.line("      p[0] = t%d[0];", n.id);
      else for (int q = 0; q < W / 4; ++q)
        e.line("      __builtin_nontemporal_store(f32x4{t%d[%d], t%d[%d], t%d[%d], t%d[%d]}, reinterpret_cast<f32x4*>(p) + %d);",
               n.id, 4 * q, n.id, 4 * q + 1, n.id, 4 * q + 2, n.id, 4 * q + 3, q);
    } else {
      const char* cv = n.out_dtype == FS_F16 ? "to_f16" : "to_bf16";
      e.line("      unsigned short* p = static_cast<unsigned short*>(a.out[%d]) + e0;", n.out_ordinal);
      if (W == 1) e.line("      p[0] = (unsigned short)%s(t%d[0]);", cv, n.id);
      else {
        e.line("      unsigned w[W / 2];");
        e.line("      UNROLL for (int j = 0; j < W / 2; ++j) w[j] = pack_%s(t%d[2 * j], t%d[2 * j + 1]);", cv, n.id, n.id);
        if (W == 8) e.line("      __builtin_nontemporal_store(u32x4{w[0], w[1], w[2], w[3]}, reinterpret_cast<u32x4*>(p));");
        else e.line("      __builtin_nontemporal_store(u32x2{w[0], w[1]}, reinterpret_cast<u32x2*>(p));");
      }
    }
    e.line("    }");
  }
  e.line("  }");
}

// the kernel is named after its own text, so that traces tell generated kernels apart
static std::string name_kernel(Emitter& e, std::string* kernel_name) {
  uint64_t h = 1469598103934665603ull;
  for (unsigned char c : e.s) { h ^= c; h *= 1099511628211ull; }
  char name[32];
  snprintf(name, sizeof name, "fs_ew_%08x", (unsigned)(h ^ (h >> 32)));
  *kernel_name = name;
  const std::string tag = "FS_EW_NAME";
  const size_t at = e.s.find(tag);
  e.s.replace(at, tag.size(), name);
  return e.s;
}

std::string ew_emit_source(const EwIr& ir, int* width, int* unroll, std::string* kernel_name) {
  const int W = chunk_width(ir);
  *width = W;
  *unroll = 1;
  Emitter e;
  e.s = kPreamble;
  e.line("extern \"C\" __global__ __launch_bounds__(256) void FS_EW_NAME(const Args a) {");
  emit_part(e, ir, W, "(long long)blockIdx.x", "(long long)gridDim.x", 0);
  e.line("}");
  return name_kernel(e, kernel_name);
}

std::string ew_emit_packed(const std::vector<const EwIr*>& parts, int wg, std::vector<int>* widths, std::vector<int>* blocks,
                           std::string* kernel_name) {
  Emitter e;
  e.s = kPreamble;
  e.line("// %zu independent groups packed into one launch: each owns a run of consecutive workgroups", parts.size());
  e.line("extern \"C\" __global__ __launch_bounds__(256) void FS_EW_NAME(const Args a) {");
  int first = 0, view_base = 0;
  widths->clear();
  blocks->clear();
  for (size_t q = 0; q < parts.size(); ++q) {
    const EwIr& ir = *parts[q];
    const int W = chunk_width(ir);
    const int64_t chunks = ir.n / W;
    int64_t nb = (chunks + wg - 1) / wg;
    if (nb > (1 << 20)) nb = 1 << 20;         // the loop strides over what is left
    if (nb < 1) nb = 1;
    widths->push_back(W);
    blocks->push_back((int)nb);
    char blk[64], nblk[32];
    snprintf(blk, sizeof blk, "(long long)(blockIdx.x - %du)", (unsigned)first);
    snprintf(nblk, sizeof nblk, "%lldll", (long long)nb);
    e.line("  if (blockIdx.x < %du) {", (unsigned)(first + nb));
    emit_part(e, ir, W, blk, nblk, view_base);
    e.line("    return;");
    e.line("  }");
    first += (int)nb;
    view_base += (int)ir.views.size();
  }
  e.line("}");
  return name_kernel(e, kernel_name);
}

// ---------------------------------------------------------------------------------------------

namespace {
std::mutex g_cache_mutex;
std::map<std::string, std::shared_ptr<std::vector<char>>> g_cache;
thread_local bool g_dry_run = false;
// Code objects on disk, so that a later process does not compile again what this one compiled:
// one file per generated source, named after a hash of the source and the compile options.
std::string g_disk_dir;
bool g_disk_dir_set = false;
int64_t g_stat_compiled = 0, g_stat_memory = 0, g_stat_disk = 0;
const char* const kCompileOptions[] = {"--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"};

uint64_t fnv(const std::string& text, uint64_t h) {
  for (unsigned char c : text) { h ^= c; h *= 1099511628211ull; }
  return h;
}

std::string disk_dir_locked() {
  if (!g_disk_dir_set) {
    if (const char* env = getenv("FS_KERNEL_CACHE_DIR")) g_disk_dir = env;
    g_disk_dir_set = true;
  }
  return g_disk_dir;
}

// what the file must belong to: the source, the options, the compiler's version
std::string cache_identity(const std::string& source) {
  int major = 0, minor = 0;
  (void)hiprtcVersion(&major, &minor);
  std::string id = "fs-code-object 1;hiprtc " + std::to_string(major) + "." + std::to_string(minor) + ";";
  for (const char* o : kCompileOptions) { id += o; id += ' '; }
  return id + "\n" + source;
}

std::string cache_path(const std::string& dir, const std::string& identity) {
  char name[48];
  snprintf(name, sizeof name, "/fs_%016llx.co", (unsigned long long)fnv(identity, 1469598103934665603ull));
  return dir + name;
}

// File layout: header, the identity text (source, options, compiler version), the code object.  A file is
// used only if the header is well formed, the identity text is the expected one byte for byte, and the code
// bytes match their checksum; anything else (a truncated or damaged file, a file written by another version,
// a hash collision on the name) is ignored and replaced by a fresh compile.
struct DiskHeader { char magic[8]; uint64_t identity_check; uint64_t identity_bytes; uint64_t code_bytes; uint64_t code_check; };

uint64_t fnv_bytes(const std::vector<char>& v, uint64_t h) {
  for (char c : v) { h ^= (unsigned char)c; h *= 1099511628211ull; }
  return h;
}

bool disk_load(const std::string& path, const std::string& identity, std::vector<char>* code) {
  FILE* f = fopen(path.c_str(), "rb");
  if (!f) return false;
  DiskHeader h{};
  bool ok = fread(&h, sizeof h, 1, f) == 1 && memcmp(h.magic, "FSCODE2", 8) == 0 && h.identity_bytes == identity.size() &&
            h.identity_check == fnv(identity, 0x9e3779b97f4a7c15ull) && h.code_bytes > 0 && h.code_bytes < (64u << 20);
  if (ok) {
    std::string stored(h.identity_bytes, '\0');
    ok = fread(&stored[0], 1, stored.size(), f) == stored.size() && stored == identity;
  }
  if (ok) {
    code->resize(h.code_bytes);
    ok = fread(code->data(), 1, h.code_bytes, f) == h.code_bytes && fgetc(f) == EOF &&
         fnv_bytes(*code, 0x9e3779b97f4a7c15ull) == h.code_check;
  }
  fclose(f);
  if (!ok) code->clear();
  return ok;
}

void disk_store(const std::string& path, const std::string& identity, const std::vector<char>& code) {
  char tmp[32];
  snprintf(tmp, sizeof tmp, ".tmp.%ld", (long)getpid());
  const std::string part = path + tmp;
  FILE* f = fopen(part.c_str(), "wb");
  if (!f) return;                               // an unwritable directory costs the next process a compile, nothing else
  DiskHeader h{};
  memcpy(h.magic, "FSCODE2", 8);
  h.identity_check = fnv(identity, 0x9e3779b97f4a7c15ull);
  h.identity_bytes = identity.size();
  h.code_bytes = code.size();
  h.code_check = fnv_bytes(code, 0x9e3779b97f4a7c15ull);
  const bool ok = fwrite(&h, sizeof h, 1, f) == 1 && fwrite(identity.data(), 1, identity.size(), f) == identity.size() &&
                  fwrite(code.data(), 1, code.size(), f) == code.size();
  if (fclose(f) != 0 || !ok || rename(part.c_str(), path.c_str()) != 0) (void)remove(part.c_str());
}
}  // namespace

void codegen_set_dry_run(bool on) { g_dry_run = on; }

void codegen_cache_dir(const char* dir) {
  std::lock_guard<std::mutex> lock(g_cache_mutex);
  g_disk_dir = dir ? dir : "";
  g_disk_dir_set = true;
}

void codegen_cache_drop_memory() {
  std::lock_guard<std::mutex> lock(g_cache_mutex);
  g_cache.clear();
}

void codegen_cache_stats(int64_t* compiled, int64_t* from_memory, int64_t* from_disk) {
  std::lock_guard<std::mutex> lock(g_cache_mutex);
  if (compiled) *compiled = g_stat_compiled;
  if (from_memory) *from_memory = g_stat_memory;
  if (from_disk) *from_disk = g_stat_disk;
}

bool ew_compile_source(const std::string& source, std::vector<char>* code_object, std::string* err) {
  if (g_dry_run) { code_object->clear(); return true; }     // planning only: the source exists, that is enough
  std::string dir;
  {
    std::lock_guard<std::mutex> lock(g_cache_mutex);
    auto it = g_cache.find(source);
    if (it != g_cache.end()) { *code_object = *it->second; ++g_stat_memory; return true; }
    dir = disk_dir_locked();
  }
  std::string identity, path;
  if (!dir.empty()) {
    identity = cache_identity(source);
    path = cache_path(dir, identity);
    if (disk_load(path, identity, code_object)) {
      std::lock_guard<std::mutex> lock(g_cache_mutex);
      g_cache[source] = std::make_shared<std::vector<char>>(*code_object);
      ++g_stat_disk;
      return true;
    }
  }
  hiprtcProgram prog = nullptr;
  hiprtcResult r = hiprtcCreateProgram(&prog, source.c_str(), "fs_ew.hip", 0, nullptr, nullptr);
  if (r != HIPRTC_SUCCESS) { *err = std::string("hiprtcCreateProgram: ") + hiprtcGetErrorString(r); return false; }
  // same code generation rules as the library's own kernels: gfx950 only, packed fp32 math off
  r = hiprtcCompileProgram(prog, (int)(sizeof kCompileOptions / sizeof kCompileOptions[0]), const_cast<const char**>(kCompileOptions));
  if (r != HIPRTC_SUCCESS) {
    size_t n = 0;
    std::string log;
    if (hiprtcGetProgramLogSize(prog, &n) == HIPRTC_SUCCESS && n > 1) {
      log.resize(n);
      (void)hiprtcGetProgramLog(prog, &log[0]);
    }
    *err = std::string("hiprtcCompileProgram: ") + hiprtcGetErrorString(r) + "\n" + log.substr(0, 2000);
    (void)hiprtcDestroyProgram(&prog);
    return false;
  }
  size_t bytes = 0;
  r = hiprtcGetCodeSize(prog, &bytes);
  if (r == HIPRTC_SUCCESS) {
    code_object->resize(bytes);
    r = hiprtcGetCode(prog, code_object->data());
  }
  (void)hiprtcDestroyProgram(&prog);
  if (r != HIPRTC_SUCCESS) { *err = std::string("hiprtcGetCode: ") + hiprtcGetErrorString(r); return false; }
  if (!path.empty()) disk_store(path, identity, *code_object);
  std::lock_guard<std::mutex> lock(g_cache_mutex);
  g_cache[source] = std::make_shared<std::vector<char>>(*code_object);
  ++g_stat_compiled;
  return true;
}

int ew_module_launch(EwModule* m, const std::vector<char>& code_object, const std::string& kernel_name,
                     const void* args, size_t args_bytes, int grid, int block, void* stream, std::string* err) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) { *err = "hipGetDevice failed"; return -1; }
  if (!m->function) {
    hipModule_t mod = nullptr;
    hipError_t e = hipModuleLoadData(&mod, code_object.data());
    if (e != hipSuccess) { *err = std::string("hipModuleLoadData: ") + hipGetErrorString(e); return -1; }
    hipFunction_t fn = nullptr;
    e = hipModuleGetFunction(&fn, mod, kernel_name.c_str());
    if (e != hipSuccess) { (void)hipModuleUnload(mod); *err = std::string("hipModuleGetFunction: ") + hipGetErrorString(e); return -1; }
    m->module = mod; m->function = fn; m->device = dev;
  } else if (dev != m->device) {
    *err = "plan is bound to the device of its first launch";
    return -1;
  }
  size_t sz = args_bytes;
  void* config[] = {HIP_LAUNCH_PARAM_BUFFER_POINTER, const_cast<void*>(args), HIP_LAUNCH_PARAM_BUFFER_SIZE, &sz, HIP_LAUNCH_PARAM_END};
  const hipError_t e = hipModuleLaunchKernel(static_cast<hipFunction_t>(m->function), (unsigned)grid, 1, 1, (unsigned)block, 1, 1, 0,
                                             static_cast<hipStream_t>(stream), nullptr, config);
  if (e != hipSuccess) { *err = std::string("hipModuleLaunchKernel: ") + hipGetErrorString(e); return -1; }
  return 0;
}

void ew_module_release(EwModule* m) {
  if (m->module) (void)hipModuleUnload(static_cast<hipModule_t>(m->module));
  m->module = nullptr; m->function = nullptr; m->device = -1;
}

}  // namespace fs
