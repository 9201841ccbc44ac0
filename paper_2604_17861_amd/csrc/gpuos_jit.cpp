// gpuos_jit.cpp -- operators defined at run time as native code (paper Sections 1.2 and 4.1: new
// operators are compiled while the executor runs and become callable through the operator table).
//
// A kernel that is already running cannot call into a code object that is loaded later, so the
// native code of the programs a context has defined lives in a SECOND resident worker kernel that
// is compiled here with the HIP run-time compiler: the worker loop and the elementwise execution
// paths of the library (csrc/gpuos_device.h, embedded below as text) instantiated with each program
// as a straight-line functor, one IEEE binary32 operation per instruction exactly as the
// interpreter evaluates it.  The dispatcher routes the tasks of those programs to that kernel's unit
// ring; everything else (descriptors, table, versions, dependencies, completion) is shared.
//
// This file only turns programs into a code object: source generation, compilation, and a cache of
// code objects keyed by the hash of the generated source.  Loading, launching and retiring the
// kernel is the runtime's business (gpuos_runtime.cpp).  The compiler library is looked up with
// dlopen at the first use: without it, or when anything here fails, programs stay interpreted
// (correctness never depends on this path).
#include <dlfcn.h>

#include <chrono>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/gpuos.h"
#include "gpuos_internal.h"

#ifndef GPUOS_CSRC_DIR
#error "GPUOS_CSRC_DIR (the directory of this file) must be defined by the build"
#endif
#define GPUOS_STR2(x) #x
#define GPUOS_STR(x) GPUOS_STR2(x)

// The three headers the run-time kernel is compiled from, as they are in the source tree,
// NUL-terminated, in read-only data.
asm(".pushsection .rodata\n"
    ".global gpuos_src_api\ngpuos_src_api:\n.incbin \"" GPUOS_STR(GPUOS_CSRC_DIR) "/../../include/gpuos.h\"\n.byte 0\n"
    ".global gpuos_src_internal\ngpuos_src_internal:\n.incbin \"" GPUOS_STR(GPUOS_CSRC_DIR) "/gpuos_internal.h\"\n.byte 0\n"
    ".global gpuos_src_device\ngpuos_src_device:\n.incbin \"" GPUOS_STR(GPUOS_CSRC_DIR) "/gpuos_device.h\"\n.byte 0\n"
    ".popsection\n");
extern "C" const char gpuos_src_api[];
extern "C" const char gpuos_src_internal[];
extern "C" const char gpuos_src_device[];

namespace gpuos {

namespace {

// the few entry points of the run-time compiler that are used (its own types reduced to what crosses here)
struct Rtc {
  void* lib = nullptr;
  int (*create)(void** prog, const char* src, const char* name, int n_headers, const char** headers, const char** names) = nullptr;
  int (*compile)(void* prog, int n_opts, const char** opts) = nullptr;
  int (*log_size)(void* prog, size_t* n) = nullptr;
  int (*log)(void* prog, char* dst) = nullptr;
  int (*code_size)(void* prog, size_t* n) = nullptr;
  int (*code)(void* prog, char* dst) = nullptr;
  int (*destroy)(void** prog) = nullptr;
  bool ok = false;
};

const Rtc& rtc() {
  static const Rtc r = [] {
    Rtc x;
    const char* names[3] = {std::getenv("GPUOS_HIPRTC_LIBRARY"), "libhiprtc.so.7", "libhiprtc.so"};
    for (const char* n : names) {
      if (!n || !*n) continue;
      x.lib = dlopen(n, RTLD_NOW | RTLD_LOCAL);
      if (x.lib) break;
    }
    if (!x.lib) return x;
    auto sym = [&](const char* s) { return dlsym(x.lib, s); };
    x.create = reinterpret_cast<decltype(x.create)>(sym("hiprtcCreateProgram"));
    x.compile = reinterpret_cast<decltype(x.compile)>(sym("hiprtcCompileProgram"));
    x.log_size = reinterpret_cast<decltype(x.log_size)>(sym("hiprtcGetProgramLogSize"));
    x.log = reinterpret_cast<decltype(x.log)>(sym("hiprtcGetProgramLog"));
    x.code_size = reinterpret_cast<decltype(x.code_size)>(sym("hiprtcGetCodeSize"));
    x.code = reinterpret_cast<decltype(x.code)>(sym("hiprtcGetCode"));
    x.destroy = reinterpret_cast<decltype(x.destroy)>(sym("hiprtcDestroyProgram"));
    x.ok = x.create && x.compile && x.log_size && x.log && x.code_size && x.code && x.destroy;
    return x;
  }();
  return r;
}

// one instruction as a C++ statement on the registers r0..r7: the same single IEEE operation the
// interpreter performs (csrc/gpuos_device.h, run_program_vec)
void emit_instr(std::string& out, uint32_t w, uint32_t imm_bits) {
  const uint32_t op = w & 0xffu, d = (w >> 8) & 7u, a = (w >> 16) & 7u, b = (w >> 24) & 7u;
  char A[4], B[4], D[4], buf[256];
  std::snprintf(A, sizeof(A), "r%u", a);
  std::snprintf(B, sizeof(B), "r%u", b);
  std::snprintf(D, sizeof(D), "r%u", d);
  const char* fmt = nullptr;
  switch (op) {
    case GPUOS_PC_MOV: fmt = "%s = %s;"; std::snprintf(buf, sizeof(buf), fmt, D, A); break;
    case GPUOS_PC_IMM: std::snprintf(buf, sizeof(buf), "%s = __builtin_bit_cast(float, 0x%08xu);", D, imm_bits); break;
    case GPUOS_PC_ADD: std::snprintf(buf, sizeof(buf), "%s = %s + %s;", D, A, B); break;
    case GPUOS_PC_SUB: std::snprintf(buf, sizeof(buf), "%s = %s - %s;", D, A, B); break;
    case GPUOS_PC_MUL: std::snprintf(buf, sizeof(buf), "%s = %s * %s;", D, A, B); break;
    case GPUOS_PC_DIV: std::snprintf(buf, sizeof(buf), "%s = %s / %s;", D, A, B); break;
    case GPUOS_PC_FMA: std::snprintf(buf, sizeof(buf), "%s = __builtin_fmaf(%s, %s, %s);", D, A, B, D); break;
    case GPUOS_PC_MAX: std::snprintf(buf, sizeof(buf), "%s = (%s != %s) ? %s : ((%s != %s) ? %s : (%s > %s ? %s : %s));", D, A, A, A, B, B, B, A, B, A, B); break;
    case GPUOS_PC_MIN: std::snprintf(buf, sizeof(buf), "%s = (%s != %s) ? %s : ((%s != %s) ? %s : (%s < %s ? %s : %s));", D, A, A, A, B, B, B, A, B, A, B); break;
    case GPUOS_PC_NEG: std::snprintf(buf, sizeof(buf), "%s = -%s;", D, A); break;
    case GPUOS_PC_ABS: std::snprintf(buf, sizeof(buf), "%s = __builtin_fabsf(%s);", D, A); break;
    case GPUOS_PC_RELU: std::snprintf(buf, sizeof(buf), "%s = (%s != %s) ? %s : (%s > 0.0f ? %s : 0.0f);", D, A, A, A, A, A); break;
    case GPUOS_PC_EXP: std::snprintf(buf, sizeof(buf), "%s = expf(%s);", D, A); break;
    case GPUOS_PC_SQRT: std::snprintf(buf, sizeof(buf), "%s = __builtin_sqrtf(%s);", D, A); break;
    default: std::snprintf(buf, sizeof(buf), "%s = 0.0f;", D); break;
  }
  (void)fmt;
  out += "    ";
  out += buf;
  out += "\n";
}

std::mutex g_cache_mu;
std::map<uint64_t, std::vector<char>> g_cache;     // hash of the generated source -> code object
uint64_t g_compiles = 0, g_hits = 0;

uint64_t fnv1a(const std::string& s) {
  uint64_t h = 0xcbf29ce484222325ull;
  for (unsigned char ch : s) h = (h ^ ch) * 0x100000001b3ull;
  return h;
}

}  // namespace

bool jit_compiler_available() { return rtc().ok; }

// The source of the run-time worker kernel for programs imgs[0 .. n).
std::string jit_source(const ProgramImage* imgs, uint32_t n) {
  std::string s;
  s += "// worker kernel with the context's operator programs as native code (generated)\n";
  // the run-time compiler has no <stdint.h>; its own fixed-width types live in a namespace
  s += "typedef unsigned char uint8_t; typedef signed char int8_t; typedef unsigned short uint16_t; typedef short int16_t;\n"
       "typedef unsigned int uint32_t; typedef int int32_t; typedef unsigned long long uint64_t; typedef long long int64_t;\n";
  s += "#include \"gpuos.h\"\n#include \"gpuos_internal.h\"\n#include \"gpuos_device.h\"\n";
  s += "namespace gpuos {\nconstexpr int kNativeOp = 1000;   // functor ids of the programs, beside the built-in implementation ids\n";
  char buf[256];
  for (uint32_t k = 0; k < n; ++k) {
    const ProgramImage& im = imgs[k];
    std::snprintf(buf, sizeof(buf), "template <> struct Op<kNativeOp + %u> {\n  static constexpr int N = %u;\n"
                  "  static DEV float f(float x, float y, float z, float alpha) {\n"
                  "    float r0 = x, r1 = y, r2 = z, r3 = alpha, r4 = 0.0f, r5 = 0.0f, r6 = 0.0f, r7 = 0.0f;\n", k, im.n_inputs);
    s += buf;
    for (uint32_t i = 0; i < im.n_instr; ++i) emit_instr(s, im.code[2 * i], im.code[2 * i + 1]);
    s += "    (void)r1; (void)r2; (void)r3; (void)r4; (void)r5; (void)r6; (void)r7;\n    return r0;\n  }\n};\n";
  }
  s += "struct NativeExec {\n"
       "  static DEV int32_t run(const Record* r, uint32_t impl, uint32_t chunk, float* s_red, const ProgramImage*) {\n"
       "    if (uni(r->path) == PATH_NOP) return GPUOS_OK;\n"
       "    switch (impl - GPUOS_IMPL_PROGRAM_BASE) {\n";
  for (uint32_t k = 0; k < n; ++k) {
    std::snprintf(buf, sizeof(buf), "      case %u: if (uni(r->n_inputs) != %uu) return GPUOS_E_INVAL; "
                  "run_elementwise<POL_COHERENT, kNativeOp + %u>(r, chunk, s_red); return GPUOS_OK;\n", k, imgs[k].n_inputs, k);
    s += buf;
  }
  s += "      default: return GPUOS_E_BADOP;\n    }\n  }\n};\n}  // namespace gpuos\n";
  s += "extern \"C\" __global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 8)))\n"
       "gpuos_native_worker(gpuos::WorkerArgs a, uint32_t gen) {\n"
       "  __shared__ gpuos::WorkShared sh;\n"
       "  if (blockIdx.x == 0 && threadIdx.x == 0)\n"
       "    __hip_atomic_store(&a.h->jit_alive, gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);\n"
       "  gpuos::run_worker<1, gpuos::NativeExec>(a, &sh, gen);\n}\n";
  return s;
}

// Compile the worker kernel for imgs[0 .. n) for gfx950, or fetch it from the cache.  Returns 0 and
// the code object, or -1 with the reason (compiler log included) in *err.
int jit_build(const ProgramImage* imgs, uint32_t n, std::vector<char>* code, std::string* err, double* compile_ms, bool* cache_hit) {
  if (compile_ms) *compile_ms = 0.0;
  if (cache_hit) *cache_hit = false;
  if (!rtc().ok) { if (err) *err = "the HIP run-time compiler library was not found"; return -1; }
  const std::string src = jit_source(imgs, n);
  // the key covers the embedded headers too: a library rebuilt from other sources never reuses a stale object
  const uint64_t key = fnv1a(src) ^ (fnv1a(gpuos_src_device) * 3u) ^ (fnv1a(gpuos_src_internal) * 5u);
  {
    std::lock_guard<std::mutex> lk(g_cache_mu);
    auto it = g_cache.find(key);
    if (it != g_cache.end()) {
      *code = it->second;
      ++g_hits;
      if (cache_hit) *cache_hit = true;
      return 0;
    }
  }
  const auto t0 = std::chrono::steady_clock::now();
  const Rtc& R = rtc();
  void* prog = nullptr;
  const char* headers[3] = {gpuos_src_api, gpuos_src_internal, gpuos_src_device};
  const char* names[3] = {"gpuos.h", "gpuos_internal.h", "gpuos_device.h"};
  if (R.create(&prog, src.c_str(), "gpuos_native_worker.hip", 3, headers, names) != 0) {
    if (err) *err = "hiprtcCreateProgram failed";
    return -1;
  }
  // the flags the library itself is built with: only the FMA instruction fuses; no packed fp32 instructions
  const char* opts[] = {"--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off",
                        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"};
  const int rc = R.compile(prog, (int)(sizeof(opts) / sizeof(opts[0])), opts);
  if (rc != 0) {
    size_t ln = 0;
    std::string log;
    if (R.log_size(prog, &ln) == 0 && ln > 1) { log.resize(ln); R.log(prog, &log[0]); }
    if (err) *err = "run-time compilation failed: " + log.substr(0, 2000);
    R.destroy(&prog);
    return -1;
  }
  size_t cn = 0;
  if (R.code_size(prog, &cn) != 0 || cn == 0) { R.destroy(&prog); if (err) *err = "empty code object"; return -1; }
  code->resize(cn);
  R.code(prog, code->data());
  R.destroy(&prog);
  if (compile_ms) *compile_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
  std::lock_guard<std::mutex> lk(g_cache_mu);
  g_cache[key] = *code;
  ++g_compiles;
  return 0;
}

void jit_cache_counts(uint64_t* compiles, uint64_t* hits) {
  std::lock_guard<std::mutex> lk(g_cache_mu);
  *compiles = g_compiles;
  *hits = g_hits;
}

}  // namespace gpuos
