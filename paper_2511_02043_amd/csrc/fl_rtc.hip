// Run-time compilation of attention variants that no compiled specialisation covers: the caller
// gives the score_mod (Eq. 4) and the mask predicate (the mask_mod of Sec. 2.2) as C expressions,
// and the forward kernel template is instantiated around them with hipRTC -- the nearest
// equivalent, in a hand-written library, of the paper's compiler taking an arbitrary attention
// program.  The generated kernel is the same software-pipelined bf16 kernel as the built-in
// variants; a custom mask is evaluated on every score (no tile is skipped, as in the paper's
// own kernels, Sec. 3.8).
#include <hip/hip_runtime.h>
#include <hip/hiprtc.h>

#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <tuple>
#include <vector>

#include "../../include/fl_attn.h"
#include "fl_host.hpp"
#include "fl_bwd_registry.hpp"
#include "fl_registry.hpp"

namespace {
#include "_build/fl_embedded.inc"   // kParamsHpp, kKernelHpp, kBwdHpp: the kernel headers as strings
}

struct fl_custom_variant {
  int D = 0;
  int waves = 4;                   // waves per workgroup of the instantiated kernel shape
  int aux_dtype[4] = {0, 0, 0, 0}; // element types of the arrays the expressions read (0: not used)
  unsigned mask = 0;               // mask bits the kernel was instantiated with
  bool has_mask_expr = false;      // a mask expression was given (a tile-class map can be built for it)
  bool per_head = false;           // ... and it reads g or h: the map is per (b, g, h), else per b
  std::vector<char> code;          // the compiled code object
  std::string kernel_name;         // lowered name of the instantiated kernel
  std::string map_kernel_name;     // lowered name of the tile-class pre-pass (variants with a mask expression)
  std::mutex mu;
  hipModule_t module[64] = {};     // loaded lazily, once per device
  hipFunction_t func[64] = {};
  hipFunction_t map_func[64] = {};
  // backward pass: the expressions are kept, the two backward kernels are compiled when first needed
  std::string mod_expr, grad_expr, mask_expr;
  bool has_mod = false;
  fl::BwdEntry* bwd = nullptr;
};

namespace {

// Kernel shape of the generated variants: 32 query rows per wave, 64-key tiles, two waves per SIMD; eight
// waves per workgroup at head dim 128 (the shape the compiled causal / plain kernels default to), four at 64.
constexpr int kBN = 64;
constexpr int waves_for(int D) { return D == 128 ? 8 : 4; }

// Does the expression use the identifier `name` (as a whole word)?
bool mentions(const char* e, const char* name) {
  const size_t n = strlen(name);
  auto word = [](char c) { return (c >= 'a' && c <= 'z') || (c >= 'A' && c <= 'Z') || (c >= '0' && c <= '9') || c == '_'; };
  for (const char* c = e; *c; ++c)
    if (strncmp(c, name, n) == 0 && (c == e || !word(c[-1])) && !word(c[n])) return true;
  return false;
}

bool expression_ok(const char* e) {
  // one C expression: no statement separators, braces, preprocessor lines or string literals
  for (const char* c = e; *c; ++c)
    if (*c == ';' || *c == '{' || *c == '}' || *c == '#' || *c == '"' || *c == '\\' || *c == '\n') return false;
  return true;
}


// Compiles `src` (which instantiates the kernels named by the expressions `insts`) for gfx950 with the
// library's own flags; returns the code object and the lowered kernel names.
fl_status compile_program(const std::string& src, const std::vector<std::string>& insts, const char* what,
                          std::vector<char>* code, std::vector<std::string>* kernel_names) {
  const char* headers[] = {kParamsHpp, kKernelHpp, kBwdHpp};
  const char* names[] = {"fl_params.hpp", "fl_kernel_bf16.hpp", "fl_bwd_bf16.hpp"};
  hiprtcProgram prog;
  if (hiprtcCreateProgram(&prog, src.c_str(), "fl_variant.hip", 3, headers, names) != HIPRTC_SUCCESS)
    return fl::host::fail(FL_ERR_LAUNCH, "hiprtcCreateProgram failed");
  std::vector<std::string> exprs;
  for (const std::string& i : insts) exprs.push_back("&" + i);
  for (const std::string& e : exprs) hiprtcAddNameExpression(prog, e.c_str());
  // gfx950 only, packed fp32 instructions off
  const char* opts[] = {"--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"};
  const hiprtcResult r = hiprtcCompileProgram(prog, (int)(sizeof(opts) / sizeof(opts[0])), opts);
  if (r != HIPRTC_SUCCESS) {
    size_t n = 0;
    hiprtcGetProgramLogSize(prog, &n);
    std::string log(n, 0);
    if (n) hiprtcGetProgramLog(prog, &log[0]);
    // the first error line is what the caller needs; the detail buffer keeps its head
    const size_t at = log.find("error:");
    fl_status st = fl::host::fail(FL_ERR_DESC, "%s: %.300s", what, at == std::string::npos ? log.c_str() : log.c_str() + at);
    hiprtcDestroyProgram(&prog);
    return st;
  }
  size_t cs = 0;
  hiprtcGetCodeSize(prog, &cs);
  code->resize(cs);
  hiprtcGetCode(prog, code->data());
  kernel_names->clear();
  for (const std::string& e : exprs) {
    const char* lowered = nullptr;
    if (hiprtcGetLoweredName(prog, e.c_str(), &lowered) != HIPRTC_SUCCESS || lowered == nullptr) {
      hiprtcDestroyProgram(&prog);
      return fl::host::fail(FL_ERR_LAUNCH, "no lowered kernel name");
    }
    kernel_names->push_back(lowered);
  }
  hiprtcDestroyProgram(&prog);
  return FL_OK;
}

fl_status compile_instance(const std::string& src, const char* inst, const char* what, std::vector<char>* code,
                           std::string* kernel_name) {
  std::vector<std::string> names;
  const fl_status st = compile_program(src, {inst}, what, code, &names);
  if (st == FL_OK) *kernel_name = names[0];
  return st;
}

// A code object loaded lazily, once per device.
struct LoadedKernel {
  std::vector<char> code;
  std::string kernel_name;
  std::mutex mu;
  hipModule_t module[64] = {};
  hipFunction_t func[64] = {};
  hipError_t get(hipFunction_t* f) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (func[dev] == nullptr) {
      if ((e = hipModuleLoadData(&module[dev], code.data())) != hipSuccess) return e;
      if ((e = hipModuleGetFunction(&func[dev], module[dev], kernel_name.c_str())) != hipSuccess) return e;
    }
    *f = func[dev];
    return hipSuccess;
  }
};

struct JitForward {
  LoadedKernel k;
  fl::KernelEntry entry;
  int nthreads;
};

}  // namespace

namespace fl {

const KernelEntry* jit_forward_entry(const JitRequest& r) {
  typedef std::tuple<int, int, int, uint32_t, int, bool, uint32_t, bool, bool, int> Key;
  static std::mutex mu;
  static std::map<Key, JitForward*> cache;        // entries live until the process ends
  const Key key(r.D, r.DV, r.mod, r.mask, r.nbias, r.diff, r.epi, r.paged, r.wide, r.pack);
  std::lock_guard<std::mutex> lock(mu);            // one compilation at a time; a hit only takes the lookup
  auto it = cache.find(key);
  if (it != cache.end()) return it->second != nullptr ? &it->second->entry : nullptr;
  // Shape of the generated kernels: one 32-row block per wave, two waves per SIMD; 4 waves (8 for the two
  // softmax streams of the differential variant); 64-key tiles unless the rings would pass 64 KiB of LDS
  // (a launch through the module API gets no more than that).
  const int nw = (r.diff || r.wide) ? 8 : 4;
  const int ns = r.diff ? 2 : 1;
  int bn = 64;
  if (2 * bn * 2 * (ns * r.D + r.DV) > 65536) bn = 32;
  const int lds = 2 * bn * 2 * (ns * r.D + r.DV);
  const int xch = r.diff ? (nw / 2) * 64 * (r.DV / 32) * 16 * 4 : 0;
  char inst[320];
  snprintf(inst, sizeof(inst), "fl::fwd_bf16_kernel<fl::Bf16Cfg<%d, %d, %d, 1, %d, 2, %d, %uu, %d, %s, %uu, 2, %s, %d>>", r.D, r.DV, nw, bn,
           r.mod, r.mask, r.nbias, r.diff ? "true" : "false", r.epi, r.paged ? "true" : "false", r.pack);
  std::string src = "#include \"fl_kernel_bf16.hpp\"\ntemplate __global__ void ";
  src += inst;
  src += "(const fl::FwdParams);\n";
  JitForward* j = new JitForward;
  if (compile_instance(src, inst, "run-time specialisation does not compile", &j->k.code, &j->k.kernel_name) != FL_OK ||
      (lds > xch ? lds : xch) > 65536) {
    delete j;
    cache[key] = nullptr;                          // do not try again
    return nullptr;
  }
  j->nthreads = nw * 64;
  j->entry = KernelEntry{KernelKey{1, r.D, r.DV, r.mod, (int)r.mask, r.nbias, r.diff ? 1 : 0, (int)r.epi, nw, 1, bn, 2, 2, r.paged ? 1 : 0, r.pack},
                         (nw / ns) * 32 / r.pack, lds > xch ? lds : xch, nullptr, j, 65536};
  cache[key] = j;
  return &j->entry;
}

hipError_t jit_forward_launch(const KernelEntry& e, const FwdParams& p, int nblocks, hipStream_t stream) {
  JitForward* j = (JitForward*)e.jit;
  hipFunction_t f = nullptr;
  hipError_t err = j->k.get(&f);
  if (err != hipSuccess) return err;
  FwdParams copy = p;
  void* args[] = {&copy};
  return hipModuleLaunchKernel(f, (unsigned)nblocks, 1, 1, (unsigned)j->nthreads, 1, 1, (unsigned)p.lds_bytes, stream, args, nullptr);
}

namespace {
struct JitBackward {
  LoadedKernel dq, dkdv;            // one code object (held twice) with both kernels
  BwdEntry entry;
};
}  // namespace

const BwdEntry* jit_backward_entry(int D, int mod, uint32_t mask, int nbias, BwdLaunchFn prep, BwdLaunchFn reduce) {
  typedef std::tuple<int, int, uint32_t, int> Key;
  static std::mutex mu;
  static std::map<Key, JitBackward*> cache;       // entries live until the process ends
  const Key key(D, mod, mask, nbias);
  std::lock_guard<std::mutex> lock(mu);            // one compilation at a time; a hit only takes the lookup
  auto it = cache.find(key);
  if (it != cache.end()) return it->second != nullptr ? &it->second->entry : nullptr;
  // Shapes: the dQ kernel streams 64-key tiles at two waves per SIMD; the dK/dV kernel is the plain one (four waves,
  // 64-row tiles), two waves per SIMD at head dim 64 and one at 128.  Their LDS is declared statically in the
  // generated code (FL_LDS_STATIC): a launch through the module API cannot ask for more than 64 KiB dynamically.
  const int bn_k = 64, wpe_k = D == 128 ? 1 : 2;
  char cq[160], ck[160];
  snprintf(cq, sizeof(cq), "fl::BwdCfg<%d, %d, %uu, 64, 2, %d>", D, mod, mask, nbias);
  snprintf(ck, sizeof(ck), "fl::BwdCfg<%d, %d, %uu, %d, %d, %d>", D, mod, mask, bn_k, wpe_k, nbias);
  const std::string iq = std::string("fl::bwd_dq_kernel<") + cq + ">", ik = std::string("fl::bwd_dkdv_kernel<") + ck + ">";
  std::string src = "#define FL_LDS_STATIC 1\n#include \"fl_bwd_bf16.hpp\"\n";
  src += "template __global__ void " + iq + "(const fl::BwdParams);\n";
  src += "template __global__ void " + ik + "(const fl::BwdParams);\n";
  JitBackward* j = new JitBackward;
  std::vector<std::string> names;
  if (compile_program(src, {iq, ik}, "run-time backward specialisation does not compile", &j->dq.code, &names) != FL_OK) {
    delete j;
    cache[key] = nullptr;                          // do not try again
    return nullptr;
  }
  j->dkdv.code = j->dq.code;
  j->dq.kernel_name = names[0];
  j->dkdv.kernel_name = names[1];
  j->entry = BwdEntry{BwdKey{D, mod, (int)mask, nbias}, 128, prep, nullptr, nullptr, reduce, j};
  cache[key] = j;
  return &j->entry;
}

hipError_t jit_backward_launch(const BwdEntry& e, int which, const BwdParams& p, int nblocks, hipStream_t stream) {
  JitBackward* j = (JitBackward*)e.jit;
  hipFunction_t f = nullptr;
  hipError_t err = (which == 0 ? j->dq : j->dkdv).get(&f);
  if (err != hipSuccess) return err;
  BwdParams copy = p;
  void* args[] = {&copy};
  return hipModuleLaunchKernel(f, (unsigned)nblocks, 1, 1, 256, 1, 1, 0, stream, args, nullptr);
}

BwdEntry* jit_backward_wrap(const std::vector<char>& code, const std::string& dq_name, const std::string& dkdv_name, int D, int mod,
                            uint32_t mask, BwdLaunchFn prep, BwdLaunchFn reduce) {
  JitBackward* j = new JitBackward;
  j->dq.code = code;
  j->dkdv.code = code;
  j->dq.kernel_name = dq_name;
  j->dkdv.kernel_name = dkdv_name;
  j->entry = BwdEntry{BwdKey{D, mod, (int)mask, 0}, 128, prep, nullptr, nullptr, reduce, j};
  return &j->entry;
}

void jit_backward_release(BwdEntry* e) {
  if (e == nullptr) return;
  JitBackward* j = (JitBackward*)e->jit;
  for (LoadedKernel* k : {&j->dq, &j->dkdv})
    for (int d = 0; d < 64; ++d)
      if (k->module[d] != nullptr) (void)hipModuleUnload(k->module[d]);
  delete j;
}

}  // namespace fl

extern "C" {

fl_status fl_compile_variant(const char* score_mod_expr, const char* mask_expr, uint32_t base_mask, int D,
                             fl_custom_variant** handle) {
  return fl_compile_variant_aux(score_mod_expr, mask_expr, base_mask, D, nullptr, handle);
}

fl_status fl_compile_variant_aux(const char* score_mod_expr, const char* mask_expr, uint32_t base_mask, int D,
                                 const int32_t* aux_dtypes, fl_custom_variant** handle) {
  return fl_compile_variant_grad(score_mod_expr, nullptr, mask_expr, base_mask, D, aux_dtypes, handle);
}

// The three device functions that wrap a variant's expressions (what an expression sees besides its arguments: the
// call's sizes and the captured arrays aux0 .. aux3; bf16 arrays read as float through a one-field wrapper).
static std::string hook_source(const fl_custom_variant* v, bool with_grad) {
  std::string scope = "  const int B = fl_p.B, G = fl_p.G, H = fl_p.H, Sq = fl_p.Sq, Sk = fl_p.Sk; (void)B; (void)G; (void)H; (void)Sq; (void)Sk;\n";
  for (int n = 0; n < 4; ++n) {
    if (v->aux_dtype[n] == 0) continue;
    const char* ty = v->aux_dtype[n] == FL_I32 ? "int" : (v->aux_dtype[n] == FL_F32 ? "float" : "fl_bf16_elem");
    char line[160];
    snprintf(line, sizeof(line), "  const %s* aux%d = (const %s*)fl_p.user_aux[%d]; (void)aux%d;\n", ty, n, ty, n, n);
    scope += line;
  }
  std::string src = "struct fl_bf16_elem { unsigned short u; __device__ operator float() const { return __uint_as_float((unsigned)u << 16); } };\n";
  src += "__device__ float fl_user_score_mod(float s, int b, int g, int h, int i, int j, const fl::FwdParams& fl_p) {\n" + scope + "  return (";
  src += v->has_mod ? v->mod_expr : std::string("s");
  src += "); }\n";
  if (with_grad) {
    src += "__device__ float fl_user_score_mod_grad(float s, int b, int g, int h, int i, int j, const fl::FwdParams& fl_p) {\n" + scope + "  return (";
    src += v->grad_expr.empty() ? std::string("1.0f") : v->grad_expr;
    src += "); }\n";
  }
  src += "__device__ bool fl_user_mask(int b, int g, int h, int i, int j, const fl::FwdParams& fl_p) {\n" + scope + "  return (";
  src += v->has_mask_expr ? v->mask_expr : std::string("false");
  src += "); }\n";
  return src;
}

// The two backward kernels of a variant, compiled when its backward pass is first asked for.
static fl_status compile_backward(fl_custom_variant* v) {
  std::lock_guard<std::mutex> lock(v->mu);
  if (v->bwd != nullptr) return FL_OK;
  const int mod = v->has_mod ? fl::kModCustom : fl::kModNone;
  char cq[160], ck[160];
  snprintf(cq, sizeof(cq), "fl::BwdCfg<%d, %d, %uu, 64, 2, 0>", v->D, mod, v->mask);
  snprintf(ck, sizeof(ck), "fl::BwdCfg<%d, %d, %uu, 64, %d, 0>", v->D, mod, v->mask, v->D == 128 ? 1 : 2);
  const std::string iq = std::string("fl::bwd_dq_kernel<") + cq + ">", ik = std::string("fl::bwd_dkdv_kernel<") + ck + ">";
  std::string src = "#define FL_LDS_STATIC 1\n#include \"fl_bwd_bf16.hpp\"\n" + hook_source(v, true);
  src += "template __global__ void " + iq + "(const fl::BwdParams);\n";
  src += "template __global__ void " + ik + "(const fl::BwdParams);\n";
  std::vector<char> code;
  std::vector<std::string> names;
  const fl_status st = compile_program(src, {iq, ik}, "backward pass of the variant does not compile", &code, &names);
  if (st != FL_OK) return st;
  int n = 0;
  const fl::BwdEntry* tab = v->D == 128 ? fl::entries_bwd128(&n) : fl::entries_bwd64(&n);
  v->bwd = fl::jit_backward_wrap(code, names[0], names[1], v->D, mod, v->mask, tab[0].prep, tab[0].reduce);
  return FL_OK;
}

fl_status fl_compile_variant_grad(const char* score_mod_expr, const char* score_mod_grad_expr, const char* mask_expr,
                                  uint32_t base_mask, int D, const int32_t* aux_dtypes, fl_custom_variant** handle) {
  fl::host::clear_detail();
  if (handle == nullptr) return fl::host::fail(FL_ERR_NULL, "handle is NULL");
  *handle = nullptr;
  if (D != 64 && D != 128) return fl::host::fail(FL_ERR_UNSUPPORTED, "custom variants are built for head dims 64 and 128");
  if (score_mod_expr == nullptr && mask_expr == nullptr) return fl::host::fail(FL_ERR_DESC, "neither a score_mod nor a mask expression");
  if (base_mask & ~(uint32_t)(FL_MASK_CAUSAL | FL_MASK_WINDOW | FL_MASK_PREFIX))
    return fl::host::fail(FL_ERR_DESC, "base_mask takes FL_MASK_CAUSAL, FL_MASK_WINDOW and FL_MASK_PREFIX");
  if ((base_mask & FL_MASK_PREFIX) && (base_mask & (FL_MASK_CAUSAL | FL_MASK_WINDOW)))
    return fl::host::fail(FL_ERR_DESC, "FL_MASK_PREFIX excludes FL_MASK_CAUSAL and FL_MASK_WINDOW");
  if (base_mask & FL_MASK_WINDOW) base_mask |= FL_MASK_CAUSAL;
  if ((score_mod_expr && !expression_ok(score_mod_expr)) || (mask_expr && !expression_ok(mask_expr)) ||
      (score_mod_grad_expr && !expression_ok(score_mod_grad_expr)))
    return fl::host::fail(FL_ERR_DESC, "an expression may not contain ; { } # \" \\ or a line break");
  if (score_mod_grad_expr != nullptr && score_mod_expr == nullptr)
    return fl::host::fail(FL_ERR_DESC, "a derivative expression without a score_mod expression");

  int adt[4] = {0, 0, 0, 0};
  for (int n = 0; n < 4 && aux_dtypes != nullptr; ++n) {
    adt[n] = aux_dtypes[n];
    if (adt[n] != 0 && adt[n] != FL_BF16 && adt[n] != FL_F32 && adt[n] != FL_I32)
      return fl::host::fail(FL_ERR_DTYPE, "aux_dtypes[%d] = %d: 0 (unused), FL_BF16, FL_F32 or FL_I32", n, adt[n]);
  }

  const int mod = score_mod_expr ? fl::kModCustom : fl::kModNone;
  const unsigned mask = (mask_expr ? fl::kMaskCustom : 0u) | base_mask;
  char inst[256];
  snprintf(inst, sizeof(inst), "fl::fwd_bf16_kernel<fl::Bf16Cfg<%d, %d, %d, 1, %d, 2, %d, %uu, 0, false, 0u>>", D, D, waves_for(D), kBN, mod, mask);
  fl_custom_variant* v = new fl_custom_variant;
  v->D = D;
  v->waves = waves_for(D);
  for (int n = 0; n < 4; ++n) v->aux_dtype[n] = adt[n];
  v->mask = mask;
  v->has_mod = score_mod_expr != nullptr;
  v->has_mask_expr = mask_expr != nullptr;
  v->per_head = mask_expr != nullptr && (mentions(mask_expr, "h") || mentions(mask_expr, "g"));
  if (score_mod_expr) v->mod_expr = score_mod_expr;
  if (score_mod_grad_expr) v->grad_expr = score_mod_grad_expr;
  if (mask_expr) v->mask_expr = mask_expr;
  bool captures = false;
  for (int n = 0; n < 4; ++n) captures = captures || adt[n] != 0;
  std::string src = std::string("#define FL_USER_CLAMP ") + (captures ? "1" : "0") + "\n#include \"fl_kernel_bf16.hpp\"\n" + hook_source(v, false);
  src += "template __global__ void ";
  src += inst;
  src += "(const fl::FwdParams);\n";
  std::vector<std::string> insts = {inst};
  if (mask_expr != nullptr) {                      // the pre-pass that classifies tiles under this mask
    char minst[128];
    snprintf(minst, sizeof(minst), "fl::block_map_kernel<%uu, %d>", mask, kBN);
    src += std::string("template __global__ void ") + minst + "(const fl::FwdParams, unsigned char*, unsigned int*);\n";
    insts.push_back(minst);
  }

  std::vector<std::string> names;
  fl_status st = compile_program(src, insts, "expression does not compile", &v->code, &names);
  // a derivative expression is given by callers who want the backward pass: its kernels are compiled now, so that an
  // error in that expression is reported here
  if (st == FL_OK && score_mod_grad_expr != nullptr) st = compile_backward(v);
  if (st != FL_OK) {
    delete v;
    return st;
  }
  v->kernel_name = names[0];
  if (names.size() > 1) v->map_kernel_name = names[1];
  *handle = v;
  return FL_OK;
}

void fl_release_variant(fl_custom_variant* v) {
  if (v == nullptr) return;
  for (int d = 0; d < 64; ++d)
    if (v->module[d] != nullptr) (void)hipModuleUnload(v->module[d]);
  fl::jit_backward_release(v->bwd);
  delete v;
}

fl_status fl_attn_fwd_custom(fl_custom_variant* v, const fl_tensor* q, const fl_tensor* k, const fl_tensor* vv, float scale,
                             int32_t window, int32_t prefix_len, fl_tensor* out, fl_tensor* lse, void* stream_v) {
  return fl_attn_fwd_custom_aux(v, q, k, vv, scale, window, prefix_len, nullptr, out, lse, stream_v);
}

// Workspace of the tile-class map of a call: one class byte per (32-row query block, 64-key tile), rows of a tile padded to
// 8 blocks; then, while they stay under 1 GiB, 64 words of hidden-score bits per block (one per lane of the wave that owns
// the block in the attention kernel).  Beyond that size the attention kernel evaluates the expression on partly visible tiles.
struct MapLayout {
  int64_t blocks;
  size_t off_bits, bits_bytes, total;
};
static MapLayout map_layout(const fl_custom_variant* v, int64_t B, int64_t G, int64_t H, int64_t Sq, int64_t Sk) {
  const int64_t nqb8 = ((Sq + 31) / 32 + 7) / 8 * 8, nkt = (Sk + kBN - 1) / kBN;
  MapLayout L;
  L.blocks = (v->per_head ? B * G * H : B) * nkt * nqb8;
  L.off_bits = ((size_t)L.blocks + 255) / 256 * 256;
  L.bits_bytes = (size_t)L.blocks * 256 <= ((size_t)1 << 30) ? (size_t)L.blocks * 256 : 0;
  L.total = L.off_bits + L.bits_bytes;
  return L;
}

size_t fl_custom_skip_workspace_size(fl_custom_variant* v, const fl_tensor* q, const fl_tensor* k) {
  if (v == nullptr || q == nullptr || k == nullptr || !v->has_mask_expr) return 0;
  if (q->size[0] < 0 || q->size[1] < 0 || q->size[2] < 0 || q->size[3] < 0 || k->size[3] < 0) return 0;
  return map_layout(v, q->size[0], q->size[1], q->size[2], q->size[3], k->size[3]).total;
}

static fl_status custom_forward(fl_custom_variant* v, const fl_tensor* q, const fl_tensor* k, const fl_tensor* vv, float scale,
                                int32_t window, int32_t prefix_len, const void* const* aux_ptrs, bool skip, void* workspace,
                                size_t workspace_bytes, fl_tensor* out, fl_tensor* lse, void* stream_v);

fl_status fl_attn_fwd_custom_aux(fl_custom_variant* v, const fl_tensor* q, const fl_tensor* k, const fl_tensor* vv, float scale,
                                 int32_t window, int32_t prefix_len, const void* const* aux_ptrs, fl_tensor* out, fl_tensor* lse,
                                 void* stream_v) {
  return custom_forward(v, q, k, vv, scale, window, prefix_len, aux_ptrs, false, nullptr, 0, out, lse, stream_v);
}

fl_status fl_attn_fwd_custom_skip(fl_custom_variant* v, const fl_tensor* q, const fl_tensor* k, const fl_tensor* vv, float scale,
                                  int32_t window, int32_t prefix_len, const void* const* aux_ptrs, void* workspace,
                                  size_t workspace_bytes, fl_tensor* out, fl_tensor* lse, void* stream_v) {
  return custom_forward(v, q, k, vv, scale, window, prefix_len, aux_ptrs, true, workspace, workspace_bytes, out, lse, stream_v);
}

static fl_status custom_forward(fl_custom_variant* v, const fl_tensor* q, const fl_tensor* k, const fl_tensor* vv, float scale,
                                int32_t window, int32_t prefix_len, const void* const* aux_ptrs, bool skip, void* workspace,
                                size_t workspace_bytes, fl_tensor* out, fl_tensor* lse, void* stream_v) {
  fl::host::clear_detail();
  if (v == nullptr || q == nullptr || k == nullptr || vv == nullptr || out == nullptr)
    return fl::host::fail(FL_ERR_NULL, "handle, q, k, v or out is NULL");
  if (!(scale > 0.f) || scale != scale || scale > 3.0e38f) return fl::host::fail(FL_ERR_DESC, "scale must be finite and > 0");
  if (q->dtype != FL_BF16) return fl::host::fail(FL_ERR_DTYPE, "custom variants take bf16 inputs");
  for (int n = 0; n < 4; ++n)
    if (v->aux_dtype[n] != 0 && (aux_ptrs == nullptr || aux_ptrs[n] == nullptr))
      return fl::host::fail(FL_ERR_AUX_MISSING, "this variant reads aux%d, which was not given", n);
  if ((v->mask & FL_MASK_WINDOW) && window < 0) return fl::host::fail(FL_ERR_DESC, "window must be >= 0");
  if ((v->mask & FL_MASK_PREFIX) && prefix_len < 0) return fl::host::fail(FL_ERR_DESC, "prefix_len must be >= 0");
  const int64_t B = q->size[0], G = q->size[1], H = q->size[2], Sq = q->size[3], D = q->size[4];
  const int64_t Hkv = k->size[2], Sk = k->size[3];
  if (D != v->D || vv->size[4] != v->D) return fl::host::fail(FL_ERR_SHAPE, "this variant was compiled for head dim %d", v->D);
  if (B < 0 || G < 0 || H < 0 || Sq < 0 || Sk <= 0) return fl::host::fail(FL_ERR_SHAPE, "negative size or no keys");
  if (Sq > 0x7fffff00LL || Sk > 0x7fffff00LL || B * G * H > 0x7fffffffLL) return fl::host::fail(FL_ERR_SHAPE, "size too large");
  if (Hkv <= 0 || H % Hkv != 0)
    if (H != 0) return fl::host::fail(FL_ERR_SHAPE, "k heads must divide q heads");
  if (B == 0 || G == 0 || H == 0 || Sq == 0) return FL_OK;
  const int64_t qsz[5] = {B, G, H, Sq, D}, ksz[5] = {B, G, Hkv, Sk, D};
  fl_status st;
  if ((st = fl::host::check_data_tensor(q, "q", FL_BF16, qsz)) != FL_OK) return st;
  if ((st = fl::host::check_data_tensor(k, "k", FL_BF16, ksz)) != FL_OK) return st;
  if ((st = fl::host::check_data_tensor(vv, "v", FL_BF16, ksz)) != FL_OK) return st;
  if (out->dtype != FL_BF16 && out->dtype != FL_F32) return fl::host::fail(FL_ERR_DTYPE, "out dtype %d", out->dtype);
  if ((st = fl::host::check_data_tensor(out, "out", out->dtype, qsz)) != FL_OK) return st;
  const bool want_lse = lse != nullptr && lse->ptr != nullptr;
  if (want_lse) {
    if (lse->dtype != FL_F32) return fl::host::fail(FL_ERR_DTYPE, "lse must be f32");
    const int64_t lsz[5] = {B, G, H, Sq, 1};
    for (int a = 0; a < 5; ++a)
      if (lse->size[a] != lsz[a]) return fl::host::fail(FL_ERR_SHAPE, "lse size[%d]", a);
    if (Sq > 1 && lse->stride[3] != 1) return fl::host::fail(FL_ERR_STRIDE, "lse must be contiguous along Sq");
  }

  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= 64) return fl::host::fail(FL_ERR_LAUNCH, "hipGetDevice: %s", hipGetErrorString(e));
  {
    std::lock_guard<std::mutex> lock(v->mu);
    if (v->func[dev] == nullptr) {
      if ((e = hipModuleLoadData(&v->module[dev], v->code.data())) != hipSuccess)
        return fl::host::fail(FL_ERR_LAUNCH, "hipModuleLoadData: %s", hipGetErrorString(e));
      if ((e = hipModuleGetFunction(&v->func[dev], v->module[dev], v->kernel_name.c_str())) != hipSuccess)
        return fl::host::fail(FL_ERR_LAUNCH, "hipModuleGetFunction(%s): %s", v->kernel_name.c_str(), hipGetErrorString(e));
      if (!v->map_kernel_name.empty() &&
          (e = hipModuleGetFunction(&v->map_func[dev], v->module[dev], v->map_kernel_name.c_str())) != hipSuccess)
        return fl::host::fail(FL_ERR_LAUNCH, "hipModuleGetFunction(%s): %s", v->map_kernel_name.c_str(), hipGetErrorString(e));
    }
  }

  fl::FwdParams p;
  memset(&p, 0, sizeof(p));
  p.q = fl::host::make_view(q);
  p.k = fl::host::make_view(k);
  p.v = fl::host::make_view(vv);
  p.out = fl::host::make_view(out);
  if (want_lse) {
    p.lse = (float*)lse->ptr;
    p.lse_sb = lse->size[0] > 1 ? lse->stride[0] : 0;
    p.lse_sg = lse->size[1] > 1 ? lse->stride[1] : 0;
    p.lse_sh = lse->size[2] > 1 ? lse->stride[2] : 0;
  }
  p.B = (int)B; p.G = (int)G; p.H = (int)H; p.Hkv = (int)Hkv; p.Sq = (int)Sq; p.Sk = (int)Sk;
  p.D = (int)D; p.Dv = (int)D;
  p.scale = scale;
  p.window = (int64_t)window > (Sq > Sk ? Sq : Sk) ? (int32_t)(Sq > Sk ? Sq : Sk) : window;   // keeps i - window clear of int32 overflow
  p.prefix = prefix_len;
  p.out_f32 = out->dtype == FL_F32;
  for (int n = 0; n < 4; ++n) p.user_aux[n] = (aux_ptrs != nullptr && v->aux_dtype[n] != 0) ? aux_ptrs[n] : nullptr;
  const int kBM = 32 * v->waves;
  p.n_qtiles = (int)((Sq + kBM - 1) / kBM);
  p.lds_bytes = 4 * kBN * (int)D * 2;              // K ring and V ring of two 64-key tiles each
  const int64_t nbh = B * G * H;
  p.order = nbh % 8 == 0 ? 1 : 0;
  // under a causal / prefix base mask without a window a workgroup takes a long and a short q-tile
  const bool tri = (v->mask & (FL_MASK_CAUSAL | FL_MASK_PREFIX)) != 0 && (v->mask & FL_MASK_WINDOW) == 0;
  p.pair = tri && nbh * ((p.n_qtiles + 1) / 2) >= 512;
  const int64_t nblocks = nbh * (p.pair ? (p.n_qtiles + 1) / 2 : p.n_qtiles);
  if (nblocks > 0x7fffffffLL) return fl::host::fail(FL_ERR_SHAPE, "too many workgroups");
  if (skip && v->has_mask_expr) {
    // the pre-pass: the mask once per score, one class byte per (32-row block, 64-key tile); the kernel then passes over
    // tiles with nothing visible and skips the per-score mask on tiles where everything is
    const MapLayout ML = map_layout(v, B, G, H, Sq, Sk);
    if (workspace == nullptr || workspace_bytes < ML.total)
      return fl::host::fail(FL_ERR_WORKSPACE, "workspace needs %zu bytes, got %zu", ML.total, workspace ? workspace_bytes : (size_t)0);
    if (((uintptr_t)workspace) % 16 != 0) return fl::host::fail(FL_ERR_ALIGN, "workspace not 16-byte aligned");
    p.block_map = (const unsigned char*)workspace;
    p.block_bits = ML.bits_bytes != 0 ? (const uint32_t*)((const char*)workspace + ML.off_bits) : nullptr;
    p.map_nqb8 = (int)(((Sq + 31) / 32 + 7) / 8 * 8);
    p.map_nkt = (int)((Sk + kBN - 1) / kBN);
    p.map_per_head = v->per_head ? 1 : 0;
    const int64_t mblocks = (v->per_head ? nbh : B) * p.map_nqb8 * ((p.map_nkt + 3) / 4);
    if (mblocks > 0x7fffffffLL) return fl::host::fail(FL_ERR_SHAPE, "too many tiles to classify");
    unsigned char* map = (unsigned char*)workspace;
    uint32_t* bits = (uint32_t*)p.block_bits;
    void* margs[] = {&p, &map, &bits};
    e = hipModuleLaunchKernel(v->map_func[dev], (unsigned)mblocks, 1, 1, 256, 1, 1, 0, (hipStream_t)stream_v, margs, nullptr);
    if (e != hipSuccess) return fl::host::fail(FL_ERR_LAUNCH, "tile-class pre-pass launch: %s", hipGetErrorString(e));
  }
  void* args[] = {&p};
  e = hipModuleLaunchKernel(v->func[dev], (unsigned)nblocks, 1, 1, (unsigned)v->waves * 64, 1, 1, (unsigned)p.lds_bytes, (hipStream_t)stream_v, args, nullptr);
  if (e != hipSuccess) return fl::host::fail(FL_ERR_LAUNCH, "custom variant launch: %s", hipGetErrorString(e));
  return FL_OK;
}

size_t fl_attn_bwd_custom_workspace_size(fl_custom_variant* v, const fl_tensor* q, const fl_tensor* k) {
  if (v == nullptr || q == nullptr || k == nullptr) return 0;
  fl_variant_desc d;
  memset(&d, 0, sizeof(d));
  d.struct_size = sizeof(d);
  d.scale = 1.f;
  d.mask = v->mask & (FL_MASK_CAUSAL | FL_MASK_WINDOW | FL_MASK_PREFIX);
  return fl_attn_bwd_workspace_size(q, k, &d);
}

fl_status fl_attn_bwd_custom(fl_custom_variant* v, const fl_tensor* q, const fl_tensor* k, const fl_tensor* vv, const fl_tensor* out,
                             const fl_tensor* dout, const fl_tensor* lse, float scale, int32_t window, int32_t prefix_len,
                             const void* const* aux_ptrs, void* workspace, size_t workspace_bytes, fl_tensor* dq, fl_tensor* dk,
                             fl_tensor* dv, void* stream_v) {
  fl::host::clear_detail();
  if (v == nullptr) return fl::host::fail(FL_ERR_NULL, "handle is NULL");
  if (!(scale > 0.f) || scale != scale || scale > 3.0e38f) return fl::host::fail(FL_ERR_DESC, "scale must be finite and > 0");
  for (int n = 0; n < 4; ++n)
    if (v->aux_dtype[n] != 0 && (aux_ptrs == nullptr || aux_ptrs[n] == nullptr))
      return fl::host::fail(FL_ERR_AUX_MISSING, "this variant reads aux%d, which was not given", n);
  if (q != nullptr && (q->size[4] != v->D || (vv != nullptr && vv->size[4] != v->D)))
    return fl::host::fail(FL_ERR_SHAPE, "this variant was compiled for head dim %d", v->D);
  fl_status st = compile_backward(v);
  if (st != FL_OK) return st;
  // the structural part of the variant as a descriptor: the backward call checks tensors, sizes the launches and fills the
  // parameter block from it; the kernels are the variant's own
  fl_variant_desc d;
  memset(&d, 0, sizeof(d));
  d.struct_size = sizeof(d);
  d.scale = scale;
  d.mask = v->mask & (FL_MASK_CAUSAL | FL_MASK_WINDOW | FL_MASK_PREFIX);
  d.window = (d.mask & FL_MASK_WINDOW) ? window : 0;
  d.prefix_len = (d.mask & FL_MASK_PREFIX) ? prefix_len : 0;
  fl_aux a;
  memset(&a, 0, sizeof(a));
  a.struct_size = sizeof(a);
  a.workspace = workspace;
  a.workspace_bytes = workspace_bytes;
  const void* ptrs[4];
  for (int n = 0; n < 4; ++n) ptrs[n] = (aux_ptrs != nullptr && v->aux_dtype[n] != 0) ? aux_ptrs[n] : nullptr;
  return fl::backward_call(q, k, vv, out, dout, lse, &d, &a, dq, dk, dv, stream_v, v->bwd, ptrs);
}

}  // extern "C"
