// gpuos_device.h -- device code shared by the library's own kernels (gpuos_kernels.hip) and by the
// worker kernels that are compiled at run time for operators defined as programs (the source of
// this file is embedded in the library for that): memory access policy, element conversions, the
// operator library, the execution paths, the chunk executor and the worker loop.  Device code only;
// compiles under hipcc and under the run-time compiler.
#pragma once
#if !defined(__HIPCC_RTC__)
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/gpuos.h"
#endif
#include "gpuos_internal.h"

namespace gpuos {


#define SC_AGENT __HIP_MEMORY_SCOPE_AGENT
#define SC_SYSTEM __HIP_MEMORY_SCOPE_SYSTEM

#define DEV __device__ __forceinline__
// The per-path executors are real functions (not inlined into the worker loop): each gets a
// register allocation of its own, so the streaming loops do not inherit the worker loop's live values.
#define PATHFN __device__ __attribute__((noinline))

// ---------------------------------------------------------------------------
// memory access policy
//
// The persistent kernel never reaches a kernel boundary, and the 8 XCDs have
// one L2 each that are not coherent with each other for ordinary accesses.
// Agent-scope acquire / release fences would make a task's data visible, but
// they write back / invalidate a whole L2 on every chunk, which costs more than
// half of the HBM bandwidth when a thousand workgroups do it.  Instead every
// access to task data, descriptors and work units made by the persistent
// kernel carries the system-scope cache policy (sc0 sc1: stores write through
// to memory, loads do not hit stale lines), plus nt on the 16-byte streaming
// accesses.  With that, "release" is: wait until this wave's stores are
// acknowledged (s_waitcnt), then publish with a relaxed atomic store; "acquire"
// is: observe the flag with a relaxed atomic load, then read with the same
// policy.  No L2-wide maintenance happens in the steady state.
//
// 16-byte accesses go through buffer instructions whose resource is rebased to
// the chunk being processed: the hardware bounds-checks them (out-of-range
// loads return 0, stores are dropped).  The ordinary one-launch-per-task kernel
// uses POL_PLAIN (non-temporal, kernel-boundary coherence as for any kernel).
// ---------------------------------------------------------------------------
enum { POL_PLAIN = 0, POL_COHERENT = 1 };
typedef int v4i __attribute__((ext_vector_type(4)));
typedef __amdgpu_buffer_rsrc_t rsrc_t;

DEV rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)bytes, 0x00020000);
}

template <int POL> struct Mem {
  static constexpr int AUX = POL == POL_COHERENT ? 19 : 2;     // sc0|sc1|nt  or  nt
  static DEV v4i ld16(rsrc_t r, uint32_t off) { return __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, AUX); }
  static DEV void st16(rsrc_t r, uint32_t off, v4i q) { __builtin_amdgcn_raw_buffer_store_b128(q, r, (int)off, 0, AUX); }
  static DEV void st8(rsrc_t r, uint32_t off, uint32_t w0, uint32_t w1) {
    typedef int v2i __attribute__((ext_vector_type(2)));
    const v2i q = {(int)w0, (int)w1};
    __builtin_amdgcn_raw_buffer_store_b64(q, r, (int)off, 0, AUX);
  }
  static DEV uint32_t ld4(const void* p, uint32_t i) {
    if (POL == POL_COHERENT) return __hip_atomic_load((const uint32_t*)p + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    return ((const uint32_t*)p)[i];
  }
  static DEV uint32_t ld2(const void* p, uint32_t i) {
    if (POL == POL_COHERENT) return __hip_atomic_load((const uint16_t*)p + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    return ((const uint16_t*)p)[i];
  }
  static DEV void st4(void* p, uint32_t i, uint32_t v) {
    if (POL == POL_COHERENT) __hip_atomic_store((uint32_t*)p + i, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    else ((uint32_t*)p)[i] = v;
  }
  static DEV void st2(void* p, uint32_t i, uint32_t v) {
    if (POL == POL_COHERENT) __hip_atomic_store((uint16_t*)p + i, (uint16_t)v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    else ((uint16_t*)p)[i] = (uint16_t)v;
  }
};

// This wave's stores (all write-through) have been acknowledged when this returns.
DEV void drain_stores() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // keeps the compiler from moving stores below
  __builtin_amdgcn_s_waitcnt(0);                           // vmcnt = expcnt = lgkmcnt = 0
}
DEV void order_loads() { __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup"); }
// Between lanes of ONE wavefront that hand data to each other through LDS: its LDS operations execute
// in order, so this only keeps the compiler from moving them across (and waits for the counter).
DEV void lds_wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// ---------------------------------------------------------------------------
// element conversions (fp16 / bf16 <-> fp32; RNE, denormals kept)
// ---------------------------------------------------------------------------
DEV float h2f(uint32_t b) { return (float)__builtin_bit_cast(_Float16, (uint16_t)b); }
DEV uint32_t f2h(float f) {
  // The empty asm keeps the fp32 value opaque: without it the compiler folds the producing
  // multiply / fma and this conversion into one mixed-precision instruction that rounds the
  // exact result straight to fp16 (one rounding), while the defined result is fp32 first.
  asm("" : "+v"(f));
  return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);
}
DEV float b2f(uint32_t b) { return __builtin_bit_cast(float, b << 16); }
DEV uint32_t f2b(float f) {
  // round-to-nearest-even, NaN stays a (quiet) NaN: gfx950 has the conversion in hardware
  // (v_cvt_pk_bf16_f32), which the compiler selects for this cast; done by hand it is six
  // integer operations per element, and the 16-bit paths are the ones short of ALU time
  return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)f);
}

template <int DT> struct Elem;
template <> struct Elem<GPUOS_F32> {
  static constexpr int V = 4, ES = 4;
  static DEV float get(const v4i& q, int k) {
    const int w = q[k];      // read the lane into a scalar first: bit-casting the element lvalue directly reads lane 0
    return __builtin_bit_cast(float, w);
  }
  static DEV void put(v4i& q, int k, float f) { q[k] = __builtin_bit_cast(int, f); }
  template <int POL> static DEV float load1(const void* p, uint32_t i) { return __builtin_bit_cast(float, Mem<POL>::ld4(p, i)); }
  template <int POL> static DEV void store1(void* p, uint32_t i, float f) { Mem<POL>::st4(p, i, __builtin_bit_cast(uint32_t, f)); }
  template <int POL> static DEV void copy1(void* o, const void* a, uint32_t i) { Mem<POL>::st4(o, i, Mem<POL>::ld4(a, i)); }
};
// 16-bit elements are taken out of and put into a 32-bit word as the halves of a two-element vector:
// the compiler then reads a half with the conversion instruction's own operand selector and writes
// two converted values with one pack (fp16) or one packed conversion (bf16), where shifts and
// masks on integers cost three to four operations per element.
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bfloat2_t __attribute__((ext_vector_type(2)));
DEV float opaque_f32(float f) {
  // keeps the fp32 value a value of its own: without it the compiler folds the producing multiply /
  // fma and the conversion into one mixed-precision instruction that rounds the exact result
  // straight to 16 bits (one rounding), while the defined result is fp32 first
  asm("" : "+v"(f));
  return f;
}
template <> struct Elem<GPUOS_F16> {
  static constexpr int V = 8, ES = 2;
  static DEV float get(const v4i& q, int k) {
    const int w = q[k >> 1];
    return (float)__builtin_bit_cast(half2_t, w)[k & 1];
  }
  static DEV void put(v4i& q, int k, float f) {
    const int w = q[k >> 1];
    half2_t h = __builtin_bit_cast(half2_t, w);
    h[k & 1] = (_Float16)opaque_f32(f);
    q[k >> 1] = __builtin_bit_cast(int, h);
  }
  template <int POL> static DEV float load1(const void* p, uint32_t i) { return h2f(Mem<POL>::ld2(p, i)); }
  template <int POL> static DEV void store1(void* p, uint32_t i, float f) { Mem<POL>::st2(p, i, f2h(f)); }
  template <int POL> static DEV void copy1(void* o, const void* a, uint32_t i) { Mem<POL>::st2(o, i, Mem<POL>::ld2(a, i)); }
};
template <> struct Elem<GPUOS_BF16> {
  static constexpr int V = 8, ES = 2;
  static DEV float get(const v4i& q, int k) {
    const uint32_t w = (uint32_t)q[k >> 1];
    return __builtin_bit_cast(float, (k & 1) ? (w & 0xffff0000u) : (w << 16));
  }
  static DEV void put(v4i& q, int k, float f) {
    const int w = q[k >> 1];
    bfloat2_t h = __builtin_bit_cast(bfloat2_t, w);
    h[k & 1] = (__bf16)f;
    q[k >> 1] = __builtin_bit_cast(int, h);
  }
  template <int POL> static DEV float load1(const void* p, uint32_t i) { return b2f(Mem<POL>::ld2(p, i)); }
  template <int POL> static DEV void store1(void* p, uint32_t i, float f) { Mem<POL>::st2(p, i, f2b(f)); }
  template <int POL> static DEV void copy1(void* o, const void* a, uint32_t i) { Mem<POL>::st2(o, i, Mem<POL>::ld2(a, i)); }
};

// Element i of a float tensor whose dtype is known at run time only.  Whatever the dtype, the load
// is that of the aligned 32-bit word that holds the element (same page as the element, so it
// cannot fault; for a 16-bit element the other half of the word is dropped): one form of load, no
// branch on the dtype in front of it, so that the loads of several elements or operands can be in
// flight together.
template <int POL> DEV float load_rt(const void* p, uint32_t i, uint32_t dt) {
  const uint64_t at = (uint64_t)(__UINTPTR_TYPE__)p + (uint64_t)i * (dt == GPUOS_F32 ? 4u : 2u);
  const uint32_t w = Mem<POL>::ld4((const void*)(__UINTPTR_TYPE__)(at & ~3ull), 0);
  const uint32_t h = ((uint32_t)at & 2u) ? (w >> 16) : (w & 0xffffu);
  const uint32_t m_f32 = dt == GPUOS_F32 ? ~0u : 0u, m_f16 = dt == GPUOS_F16 ? ~0u : 0u, m_bf16 = dt == GPUOS_BF16 ? ~0u : 0u;
  return __builtin_bit_cast(float, (w & m_f32) | (__builtin_bit_cast(uint32_t, h2f(h)) & m_f16) | ((h << 16) & m_bf16));
}
template <int POL> DEV void store_rt(void* p, uint32_t i, uint32_t dt, float f) {
  if (dt == GPUOS_F32) Mem<POL>::st4(p, i, __builtin_bit_cast(uint32_t, f));
  else if (dt == GPUOS_F16) Mem<POL>::st2(p, i, f2h(f));
  else Mem<POL>::st2(p, i, f2b(f));
}

// ---------------------------------------------------------------------------
// operator library (paper Section 5.2).  fp32 in, fp32 out; the caller rounds
// to the output dtype.  GELU is evaluated in fp64 in a cancellation-free form
// and rounded once: an fp32 evaluation cannot hold 2 ulp for x < 0, where
// 1 + tanh(u) and 1 + erf(u) cancel.
// ---------------------------------------------------------------------------
constexpr uint32_t kNoLoad = 0x7ffffff0u;   // a buffer offset past every resource: the load returns 0 and moves no data

template <int IMPL> struct Op;
template <> struct Op<GPUOS_IMPL_ADD> { static constexpr int N = 2; static DEV float f(float x, float y, float, float) { return x + y; } };
template <> struct Op<GPUOS_IMPL_SUB> { static constexpr int N = 2; static DEV float f(float x, float y, float, float) { return x - y; } };
template <> struct Op<GPUOS_IMPL_MUL> { static constexpr int N = 2; static DEV float f(float x, float y, float, float) { return x * y; } };
template <> struct Op<GPUOS_IMPL_DIV> { static constexpr int N = 2; static DEV float f(float x, float y, float, float) { return x / y; } };
template <> struct Op<GPUOS_IMPL_RELU> { static constexpr int N = 1; static DEV float f(float x, float, float, float) { return (x != x) ? x : (x > 0.0f ? x : 0.0f); } };
template <> struct Op<GPUOS_IMPL_EXP> { static constexpr int N = 1; static DEV float f(float x, float, float, float) { return expf(x); } };
template <> struct Op<GPUOS_IMPL_GELU_ERF> {
  static constexpr int N = 1;
  static DEV float f(float x, float, float, float) {
    const double xd = (double)x;
    return (float)(0.5 * xd * erfc(-xd * 0.70710678118654752440));
  }
};
template <> struct Op<GPUOS_IMPL_GELU_TANH> {
  static constexpr int N = 1;
  static DEV float f(float x, float, float, float) {
    const double xd = (double)x;
    const double u = 0.79788456080286535588 * (xd + 0.044715 * xd * xd * xd);
    return (float)(xd / (1.0 + exp(-2.0 * u)));
  }
};
template <> struct Op<GPUOS_IMPL_SCALE> { static constexpr int N = 1; static DEV float f(float x, float, float, float a) { return x * a; } };
template <> struct Op<GPUOS_IMPL_FMA> { static constexpr int N = 3; static DEV float f(float x, float y, float z, float) { return __builtin_fmaf(x, y, z); } };
template <> struct Op<GPUOS_IMPL_SUB_EXP> { static constexpr int N = 2; static DEV float f(float x, float y, float, float) { const float d = x - y; return expf(d); } };
template <> struct Op<GPUOS_IMPL_COPY> { static constexpr int N = 1; static DEV float f(float x, float, float, float) { return x; } };

// ---------------------------------------------------------------------------
// operator programs: elementwise operators defined at run time, interpreted.  The program of
// the chunk being executed sits in LDS (exec_program puts it there); every lane runs the same
// instruction on its own element, so opcode and register numbers are wavefront-uniform and the
// loop over the instructions is scalar control flow.  One IEEE binary32 operation per instruction.
// ---------------------------------------------------------------------------
__shared__ ProgramImage g_prog;

// internal implementation tags: "the program in LDS, taking N inputs"
enum { kImplProg1 = 201, kImplProg2 = 202, kImplProg3 = 203 };

// The same program over K elements at once: every instruction is decoded once (scalar work) and
// applied to the K elements a lane holds, so the interpreter's overhead is shared by a whole
// 16-byte vector instead of being paid per element.
template <int K>
DEV void run_program_vec(const float (&x)[K], const float (&y)[K], const float (&z)[K], float alpha, float (&o)[K]) {
  // The register file is eight separately named arrays selected by a switch on the (uniform)
  // register number: a dynamically indexed array would be placed in scratch memory.
  float r0[K], r1[K], r2[K], r3[K], r4[K], r5[K], r6[K], r7[K];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    r0[k] = x[k]; r1[k] = y[k]; r2[k] = z[k]; r3[k] = alpha;
    r4[k] = 0.f; r5[k] = 0.f; r6[k] = 0.f; r7[k] = 0.f;
  }
#define GPUOS_RF_COPY(dst, src) _Pragma("unroll") for (int k = 0; k < K; ++k) dst[k] = src[k];
#define GPUOS_RF_READ(dst, idx) switch (idx) { \
    case 0: GPUOS_RF_COPY(dst, r0) break; case 1: GPUOS_RF_COPY(dst, r1) break; \
    case 2: GPUOS_RF_COPY(dst, r2) break; case 3: GPUOS_RF_COPY(dst, r3) break; \
    case 4: GPUOS_RF_COPY(dst, r4) break; case 5: GPUOS_RF_COPY(dst, r5) break; \
    case 6: GPUOS_RF_COPY(dst, r6) break; default: GPUOS_RF_COPY(dst, r7) break; }
#define GPUOS_RF_WRITE(idx, src) switch (idx) { \
    case 0: GPUOS_RF_COPY(r0, src) break; case 1: GPUOS_RF_COPY(r1, src) break; \
    case 2: GPUOS_RF_COPY(r2, src) break; case 3: GPUOS_RF_COPY(r3, src) break; \
    case 4: GPUOS_RF_COPY(r4, src) break; case 5: GPUOS_RF_COPY(r5, src) break; \
    case 6: GPUOS_RF_COPY(r6, src) break; default: GPUOS_RF_COPY(r7, src) break; }
  const uint32_t n = __builtin_amdgcn_readfirstlane(g_prog.n_instr);
  for (uint32_t i = 0; i < n; ++i) {
    const uint32_t w = __builtin_amdgcn_readfirstlane(g_prog.code[2 * i]);
    const float imm = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(g_prog.code[2 * i + 1]));
    const uint32_t op = w & 0xffu, d = (w >> 8) & 7u, ia = (w >> 16) & 7u, ib = (w >> 24) & 7u;
    float a[K], b[K], v[K];
    GPUOS_RF_READ(a, ia)
    GPUOS_RF_READ(b, ib)
    switch (op) {
#define GPUOS_PC_CASE(code, expr) case code: _Pragma("unroll") for (int k = 0; k < K; ++k) v[k] = (expr); break;
      GPUOS_PC_CASE(GPUOS_PC_MOV, a[k])
      GPUOS_PC_CASE(GPUOS_PC_IMM, imm)
      GPUOS_PC_CASE(GPUOS_PC_ADD, a[k] + b[k])
      GPUOS_PC_CASE(GPUOS_PC_SUB, a[k] - b[k])
      GPUOS_PC_CASE(GPUOS_PC_MUL, a[k] * b[k])
      GPUOS_PC_CASE(GPUOS_PC_DIV, a[k] / b[k])
      GPUOS_PC_CASE(GPUOS_PC_MAX, (a[k] != a[k]) ? a[k] : ((b[k] != b[k]) ? b[k] : (a[k] > b[k] ? a[k] : b[k])))
      GPUOS_PC_CASE(GPUOS_PC_MIN, (a[k] != a[k]) ? a[k] : ((b[k] != b[k]) ? b[k] : (a[k] < b[k] ? a[k] : b[k])))
      GPUOS_PC_CASE(GPUOS_PC_NEG, -a[k])
      GPUOS_PC_CASE(GPUOS_PC_ABS, __builtin_fabsf(a[k]))
      GPUOS_PC_CASE(GPUOS_PC_RELU, (a[k] != a[k]) ? a[k] : (a[k] > 0.0f ? a[k] : 0.0f))
      GPUOS_PC_CASE(GPUOS_PC_EXP, expf(a[k]))
      GPUOS_PC_CASE(GPUOS_PC_SQRT, __builtin_sqrtf(a[k]))
#undef GPUOS_PC_CASE
      case GPUOS_PC_FMA: {
        float c[K];
        GPUOS_RF_READ(c, d)
#pragma unroll
        for (int k = 0; k < K; ++k) v[k] = __builtin_fmaf(a[k], b[k], c[k]);
      } break;
      default:
#pragma unroll
        for (int k = 0; k < K; ++k) v[k] = 0.f;
        break;
    }
    GPUOS_RF_WRITE(d, v)
  }
#pragma unroll
  for (int k = 0; k < K; ++k) o[k] = r0[k];
#undef GPUOS_RF_COPY
#undef GPUOS_RF_READ
#undef GPUOS_RF_WRITE
}

DEV float run_program(float x, float y, float z, float alpha) {      // one element (strided and ragged-tail paths)
  const float xs[1] = {x}, ys[1] = {y}, zs[1] = {z};
  float os[1];
  run_program_vec<1>(xs, ys, zs, alpha, os);
  return os[0];
}
template <> struct Op<kImplProg1> { static constexpr int N = 1; static DEV float f(float x, float, float, float a) { return run_program(x, 0.f, 0.f, a); } };
template <> struct Op<kImplProg2> { static constexpr int N = 2; static DEV float f(float x, float y, float, float a) { return run_program(x, y, 0.f, a); } };
template <> struct Op<kImplProg3> { static constexpr int N = 3; static DEV float f(float x, float y, float z, float a) { return run_program(x, y, z, a); } };

// The exponential when the result is going to be rounded to a 16-bit format: the hardware base-2
// exponential of x * log2(e).  Its relative error (2^-17 at the ends of the range: the product's
// rounding, times ln 2; one step of the hardware exponential on top) is far below half a step of
// either 16-bit format (2^-9, 2^-12), so the rounded result is the correctly rounded one or its
// neighbour, inside the 2 units allowed; the full-precision routine it replaces costs about twenty
// operations where this costs two (fp16) or seven (bf16).  The hardware exponential flushes results
// below fp32's normal range.  fp16 does not care (everything below 2^-25 rounds to zero there);
// bf16 shares fp32's range, so there the argument is raised by 64 and the result scaled back with an
// exact multiplication, which rounds into the subnormal range correctly.
template <int DT> DEV float exp_for_16bit(float x) {
  const float t = x * 1.44269504088896340736f;
  if (DT == GPUOS_F16) return __builtin_amdgcn_exp2f(t);
  const bool low = t < -120.0f;
  return __builtin_amdgcn_exp2f(low ? t + 64.0f : t) * (low ? 0x1.0p-64f : 1.0f);
}
// Op<IMPL> as it is evaluated when the output dtype is DT
template <int IMPL, int DT> struct OpOut : Op<IMPL> {};
template <> struct OpOut<GPUOS_IMPL_EXP, GPUOS_F16> { static constexpr int N = 1; static DEV float f(float x, float, float, float) { return exp_for_16bit<GPUOS_F16>(x); } };
template <> struct OpOut<GPUOS_IMPL_EXP, GPUOS_BF16> { static constexpr int N = 1; static DEV float f(float x, float, float, float) { return exp_for_16bit<GPUOS_BF16>(x); } };
template <> struct OpOut<GPUOS_IMPL_SUB_EXP, GPUOS_F16> { static constexpr int N = 2; static DEV float f(float x, float y, float, float) { const float d = x - y; return exp_for_16bit<GPUOS_F16>(d); } };
template <> struct OpOut<GPUOS_IMPL_SUB_EXP, GPUOS_BF16> { static constexpr int N = 2; static DEV float f(float x, float y, float, float) { const float d = x - y; return exp_for_16bit<GPUOS_BF16>(d); } };

// o[k] = f(x[k], y[k], z[k], alpha) for the K elements a lane holds: element by element for the
// built-in implementations (the compiler unrolls it back into straight code), instruction by
// instruction for a program.
template <int IMPL, int K, int DT = GPUOS_F32>
DEV void apply_vec(const float (&x)[K], const float (&y)[K], const float (&z)[K], float alpha, float (&o)[K]) {
  if (IMPL == kImplProg1 || IMPL == kImplProg2 || IMPL == kImplProg3) {
    run_program_vec<K>(x, y, z, alpha, o);
  } else {
#pragma unroll
    for (int k = 0; k < K; ++k) o[k] = OpOut<IMPL, DT>::f(x[k], y[k], z[k], alpha);
  }
}

template <int IMPL> DEV uint32_t int_op(uint32_t x, uint32_t y) {
  if (IMPL == GPUOS_IMPL_ADD) return x + y;
  if (IMPL == GPUOS_IMPL_SUB) return x - y;
  if (IMPL == GPUOS_IMPL_MUL) return x * y;
  return x;
}

DEV uint32_t uni(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }
DEV const char* uni_ptr(uint64_t p) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)p);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(p >> 32));
  return (const char*)(((uint64_t)hi << 32) | lo);
}
// Arguments of a PATHFN function arrive in vector registers and pointers arrive generic.  Both
// facts are restored on entry: values the whole workgroup shares go back to scalar registers
// (uni / uni_ptr), and a pointer known to address LDS goes back to the LDS address space (so that
// it is read with LDS instructions, not flat ones).
template <class T> DEV T* lds_arg(T* p) {
  typedef __attribute__((address_space(3))) T* lds_t;
  const uint32_t a = uni((uint32_t)(__UINTPTR_TYPE__)(lds_t)p);
  return (T*)(lds_t)(__UINTPTR_TYPE__)a;
}

// ---------------------------------------------------------------------------
// PATH_CONTIG: out[i] = f(a[i], b[i], c[i]), all operands the same dtype.
// 16 bytes per lane per access, four accesses in flight per operand.
// ---------------------------------------------------------------------------
template <int POL, int IMPL, int DT>
PATHFN void ew_contig(const Record* r_v, uint32_t begin_v, uint32_t end_v) {
  const Record* r = lds_arg(r_v);
  uint32_t begin = uni(begin_v);
  const uint32_t end = uni(end_v);
  using E = Elem<DT>;
  using M = Mem<POL>;
  constexpr int V = E::V, N = Op<IMPL>::N, U = 4;
  const char* pa = uni_ptr(r->ptr[0]);
  const char* pb = N > 1 ? uni_ptr(r->ptr[1]) : pa;
  const char* pc = N > 2 ? uni_ptr(r->ptr[2]) : pa;
  char* po = (char*)uni_ptr(r->ptr[3]);
  const float alpha = r->alpha;
  const uint32_t tid = threadIdx.x;
  if (r->rflags & RF_VEC) {
    // buffer resources rebased to this chunk; begin is a multiple of V
    const uint32_t nvec = (end - begin) / V;
    const uint32_t bytes = nvec * 16u;
    const uint64_t boff = (uint64_t)begin * E::ES;
    const rsrc_t ra = make_rsrc(pa + boff, bytes), rb = make_rsrc(pb + boff, bytes), rc = make_rsrc(pc + boff, bytes);
    const rsrc_t ro = make_rsrc(po + boff, bytes);
    uint32_t v = tid;
    for (; v + (U - 1) * kThreads < nvec; v += U * kThreads) {
      v4i qa[U], qb[U], qc[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        qa[u] = M::ld16(ra, (v + u * kThreads) * 16u);
        if (N > 1) qb[u] = M::ld16(rb, (v + u * kThreads) * 16u);
        if (N > 2) qc[u] = M::ld16(rc, (v + u * kThreads) * 16u);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        v4i q;
        if (IMPL == GPUOS_IMPL_COPY) q = qa[u];
        else {
          float xa[V], xb[V], xc[V], xo[V];
#pragma unroll
          for (int k = 0; k < V; ++k) {
            xa[k] = E::get(qa[u], k); xb[k] = N > 1 ? E::get(qb[u], k) : 0.f; xc[k] = N > 2 ? E::get(qc[u], k) : 0.f;
          }
          apply_vec<IMPL, V, DT>(xa, xb, xc, alpha, xo);
#pragma unroll
          for (int k = 0; k < V; ++k) E::put(q, k, xo[k]);
        }
        M::st16(ro, (v + u * kThreads) * 16u, q);
      }
    }
    for (; v < nvec; v += kThreads) {
      const v4i qa = M::ld16(ra, v * 16u);
      v4i qb, qc, q;
      if (N > 1) qb = M::ld16(rb, v * 16u);
      if (N > 2) qc = M::ld16(rc, v * 16u);
      if (IMPL == GPUOS_IMPL_COPY) q = qa;
      else {
        float xa[V], xb[V], xc[V], xo[V];
#pragma unroll
        for (int k = 0; k < V; ++k) {
          xa[k] = E::get(qa, k); xb[k] = N > 1 ? E::get(qb, k) : 0.f; xc[k] = N > 2 ? E::get(qc, k) : 0.f;
        }
        apply_vec<IMPL, V, DT>(xa, xb, xc, alpha, xo);
#pragma unroll
        for (int k = 0; k < V; ++k) E::put(q, k, xo[k]);
      }
      M::st16(ro, v * 16u, q);
    }
    begin += nvec * V;                                // ragged tail below
  }
  for (uint32_t i = begin + tid; i < end; i += kThreads) {
    if (IMPL == GPUOS_IMPL_COPY) E::template copy1<POL>(po, pa, i);
    else
      E::template store1<POL>(po, i, OpOut<IMPL, DT>::f(E::template load1<POL>(pa, i), N > 1 ? E::template load1<POL>(pb, i) : 0.f,
                                                 N > 2 ? E::template load1<POL>(pc, i) : 0.f, alpha));
  }
}

template <int POL, int IMPL>
PATHFN void ew_contig_int(const Record* r_v, uint32_t begin_v, uint32_t end_v) {
  const Record* r = lds_arg(r_v);
  const uint32_t begin = uni(begin_v), end = uni(end_v);
  const char* a = uni_ptr(r->ptr[0]);
  const char* b = r->n_inputs > 1 ? uni_ptr(r->ptr[1]) : a;
  char* o = (char*)uni_ptr(r->ptr[3]);
  for (uint32_t i = begin + threadIdx.x; i < end; i += kThreads)
    Mem<POL>::st4(o, i, int_op<IMPL>(Mem<POL>::ld4(a, i), Mem<POL>::ld4(b, i)));
}

// ---------------------------------------------------------------------------
// PATH_ROW2D: contiguous [R, C] output of dtype DT, C a multiple of the vector
// width; each input is a full [R, C] tensor (dtype DT), a row vector [C]
// broadcast over rows (dtype DT), or one scalar per row (any float dtype).
// ---------------------------------------------------------------------------
constexpr uint32_t kScratchFloats = 7168;   // LDS scratch per workgroup (gather staging, transpose tiles, reduction partials): 28 KB,
                                            // still below what the dispatcher's workgroup needs, so the kernel's allocation does not grow

// KIND1 >= 0: a binary operation whose first operand is a full tensor and whose second is of that
// kind (the attention chain's layouts: full + row vector, full + per-row scalar); the kinds are then
// compile-time facts and the selects and branches on them disappear.  KIND1 < 0: kinds read from
// the descriptor.
template <int POL, int IMPL, int DT, int KIND1>
PATHFN void ew_row2d(const Record* r_v, uint32_t begin_v, uint32_t end_v, float* s_v) {
  const Record* r = lds_arg(r_v);
  const uint32_t begin = uni(begin_v), end = uni(end_v);
  float* s_scratch = lds_arg(s_v);
  using E = Elem<DT>;
  using M = Mem<POL>;
  constexpr int V = E::V, N = Op<IMPL>::N;
  const uint32_t C = uni(r->size[1]);
  const char* p[3];
  uint32_t kind[3], dt[3], st0[3];
  rsrc_t rs[3];
  const uint32_t nvec = (end - begin) / V;
  const uint64_t boff = (uint64_t)begin * E::ES;
  uint32_t n_scalar = 0;
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    const int kk = k < N ? k : 0;
    p[k] = uni_ptr(r->ptr[kk]);
    kind[k] = KIND1 < 0 ? uni(r->okind[kk]) : (kk == 0 ? (uint32_t)K_FULL : (uint32_t)KIND1);
    dt[k] = uni(r->dtype[kk]);
    st0[k] = uni(r->stride[kk][0]);
    // full operands: rebased to the chunk; row vectors: the whole vector
    rs[k] = kind[k] == K_FULL ? make_rsrc(p[k] + boff, nvec * 16u) : make_rsrc(p[k], C * E::ES);
    if (k < N && kind[k] == K_ROWSCALAR) ++n_scalar;
  }
  const rsrc_t ro = make_rsrc(uni_ptr(r->ptr[3]) + boff, nvec * 16u);
  const float alpha = r->alpha;
  // Per-row scalars (x - rowmax, e / rowsum): the rows of this chunk are gathered once into LDS
  // with coalesced loads and broadcast from there; without the staging every 16-byte vector would
  // cost one more uncached 4-byte memory request.
  const uint32_t row_first = begin / C, row_cnt = (end - 1) / C - row_first + 1;
  const bool staged = n_scalar != 0 && row_cnt * n_scalar <= kScratchFloats;
  // UN vectors per thread and round, all their loads issued before the first result is needed.
  // A chunk is one or two rounds, so the round is made long (a chunk of 12K 16-bit elements is
  // exactly one) and the first round's loads leave BEFORE the row scalars are staged: the chunk
  // then pays one memory latency, not three in a row.
  constexpr int UN = (N == 2 && KIND1 != (int)K_ROWVEC) ? 6 : 4;
  // (row, column) of a thread's vectors: one division per chunk, then steps with a carry
  const uint32_t step = kThreads * V;
  const uint32_t step_rows = step / C, step_cols = step - step_rows * C;
  uint32_t row, col;
  {
    const uint32_t i = begin + threadIdx.x * V;
    row = i / C;
    col = i - row * C;
  }
  v4i q[UN][3];
  uint32_t rowu[UN];
  auto load_round = [&](uint32_t v0) {
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const uint32_t v = v0 + (uint32_t)u * kThreads;
      const bool act = v < nvec;
      rowu[u] = row;
#pragma unroll
      for (int k = 0; k < N; ++k) {
        if (kind[k] == K_FULL) q[u][k] = M::ld16(rs[k], act ? v * 16u : kNoLoad);
        else if (kind[k] == K_ROWVEC) q[u][k] = M::ld16(rs[k], act ? col * E::ES : kNoLoad);
      }
      row += step_rows;
      col += step_cols;
      if (col >= C) { col -= C; ++row; }
    }
  };
  auto compute_round = [&](uint32_t v0) {
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const uint32_t v = v0 + (uint32_t)u * kThreads;
      if (v < nvec) {
        float sc[3] = {0.f, 0.f, 0.f};
        uint32_t region = 0;
#pragma unroll
        for (int k = 0; k < N; ++k)
          if (kind[k] == K_ROWSCALAR) {
            if (staged) { sc[k] = s_scratch[region + rowu[u] - row_first]; region += row_cnt; }
            else sc[k] = load_rt<POL>(p[k], rowu[u] * st0[k], dt[k]);
          }
        v4i res;
        float xv[3][V], xo[V];
#pragma unroll
        for (int e = 0; e < V; ++e)
#pragma unroll
          for (int k = 0; k < 3; ++k) xv[k][e] = k < N ? ((kind[k] == K_ROWSCALAR) ? sc[k] : E::get(q[u][k], e)) : 0.f;
        apply_vec<IMPL, V, DT>(xv[0], xv[1], xv[2], alpha, xo);
#pragma unroll
        for (int e = 0; e < V; ++e) E::put(res, e, xo[e]);
        M::st16(ro, v * 16u, res);
      }
    }
  };
  load_round(threadIdx.x);                           // (every thread, whatever nvec: the barrier below is for all)
  if (staged) {
    uint32_t region = 0;
#pragma unroll
    for (int k = 0; k < N; ++k)
      if (kind[k] == K_ROWSCALAR) {
        for (uint32_t t = threadIdx.x; t < row_cnt; t += kThreads)
          s_scratch[region + t] = load_rt<POL>(p[k], (row_first + t) * st0[k], dt[k]);
        region += row_cnt;
      }
    __syncthreads();
  }
  compute_round(threadIdx.x);
  for (uint32_t v0 = threadIdx.x + kThreads * UN; v0 < nvec; v0 += kThreads * UN) {
    load_round(v0);
    compute_round(v0);
  }
  if (staged) __syncthreads();        // the scratch may be reused by the next chunk
}

// ---------------------------------------------------------------------------
// PATH_TILE2D: contiguous [B, R, C] output where at least one input is stored with R as its
// unit-stride dim (a transposed view).  Such an input is gathered through a 32 x 32 LDS tile:
// it is read along ITS contiguous dim (coalesced), written to LDS, and read back transposed
// (pitch 33: no bank conflicts), so neither side of the transpose touches memory with a stride.
// Row-major inputs (unit stride along C, any row pitch, including 0 for a broadcast row) are
// read directly.  Any float dtype per operand.
// ---------------------------------------------------------------------------
constexpr uint32_t kTile = 32, kTilePitch = 33;

template <int POL, int IMPL>
PATHFN void ew_tile2d(const Record* r_v, uint32_t begin_v, uint32_t end_v, float* s_v) {
  const Record* r = lds_arg(r_v);
  const uint32_t tile_begin = uni(begin_v), tile_end = uni(end_v);
  float* s_scratch = lds_arg(s_v);
  constexpr int N = Op<IMPL>::N;
  const uint32_t R = uni(r->size[1]), C = uni(r->size[2]);
  const uint32_t tr = (R + kTile - 1) / kTile, tc = (C + kTile - 1) / kTile;
  const char* p[3];
  uint32_t kind[3], dt[3], sb[3], sr[3], sc[3];
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    const int kk = k < N ? k : 0;
    p[k] = uni_ptr(r->ptr[kk]);
    kind[k] = uni(r->okind[kk]);
    dt[k] = uni(r->dtype[kk]);
    sb[k] = uni(r->stride[kk][0]); sr[k] = uni(r->stride[kk][1]); sc[k] = uni(r->stride[kk][2]);
  }
  char* po = (char*)uni_ptr(r->ptr[3]);
  const uint32_t odt = uni(r->dtype[3]);
  const float alpha = r->alpha;
  const uint32_t tid = threadIdx.x;
  uint32_t m_f32[3], m_f16[3], m_bf16[3];                  // all ones for the input's dtype
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    m_f32[k] = dt[k] == GPUOS_F32 ? ~0u : 0u;
    m_f16[k] = dt[k] == GPUOS_F16 ? ~0u : 0u;
    m_bf16[k] = dt[k] == GPUOS_BF16 ? ~0u : 0u;
  }
  for (uint32_t t = tile_begin; t < tile_end; ++t) {
    const uint32_t b = t / (tr * tc), rem = t - b * tr * tc;
    const uint32_t ti = rem / tc, tj = rem - ti * tc;
    const uint32_t r0 = ti * kTile, c0 = tj * kTile;
    // Everything the tile needs is requested first, four elements per lane and input, and used
    // afterwards: one memory latency per tile, not one per element.  A transposed input is read
    // with the lanes along r (its contiguous dim), the others along c, where they are used; a lane
    // outside the tensor reads the tile's first element instead (in bounds) and drops it.  Whatever
    // the dtype, the load is that of the aligned 32-bit word that holds the element (same page, so
    // it cannot fault; the other half of the word is dropped): one form of load for every input,
    // no branch between the requests.
    uint32_t raw[3][4], upper[3][4];
#pragma unroll
    for (int k = 0; k < N; ++k) {
      const uint32_t es = dt[k] == GPUOS_F32 ? 4u : 2u;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t idx = tid + i * kThreads, lo5 = idx & (kTile - 1), hi5 = idx / kTile;
        uint32_t off;
        if (kind[k] == K_TRANSPOSED) {
          const bool in = r0 + lo5 < R && c0 + hi5 < C;
          off = b * sb[k] + r0 + c0 * sc[k] + (in ? lo5 + hi5 * sc[k] : 0u);
        } else {
          const bool in = r0 + hi5 < R && c0 + lo5 < C;
          off = b * sb[k] + r0 * sr[k] + c0 + (in ? hi5 * sr[k] + lo5 : 0u);
        }
        const uint64_t at = (uint64_t)(__UINTPTR_TYPE__)p[k] + (uint64_t)off * es;
        upper[k][i] = (uint32_t)at & 2u;
        raw[k][i] = Mem<POL>::ld4((const void*)(__UINTPTR_TYPE__)(at & ~3ull), 0);
      }
    }
    float x[3][4];
#pragma unroll
    for (int k = 0; k < 3; ++k)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        // (masks, not branches on the dtype)
        const uint32_t w = k < N ? raw[k][i] : 0u;
        const uint32_t h = (k < N && upper[k][i]) ? (w >> 16) : (w & 0xffffu);
        const uint32_t bits = (w & m_f32[k]) | (__builtin_bit_cast(uint32_t, h2f(h)) & m_f16[k]) | ((h << 16) & m_bf16[k]);
        x[k][i] = k < N ? __builtin_bit_cast(float, bits) : 0.0f;
      }
    // the transposed operands go through LDS: written along r, read back along c
#pragma unroll
    for (int k = 0; k < N; ++k)
      if (kind[k] == K_TRANSPOSED) {
        float* tile = s_scratch + k * (kTile * kTilePitch);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const uint32_t idx = tid + i * kThreads, rr = idx & (kTile - 1), cc = idx / kTile;
          tile[cc * kTilePitch + rr] = x[k][i];
        }
      }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < N; ++k)
      if (kind[k] == K_TRANSPOSED) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const uint32_t idx = tid + i * kThreads, cc = idx & (kTile - 1), rr = idx / kTile;
          x[k][i] = s_scratch[k * (kTile * kTilePitch) + cc * kTilePitch + rr];
        }
      }
    // compute: lanes run along c (the output's contiguous dim)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t idx = tid + i * kThreads, cc = idx & (kTile - 1), rr = idx / kTile;
      if (r0 + rr < R && c0 + cc < C)
        store_rt<POL>(po, (b * R + r0 + rr) * C + c0 + cc, odt, Op<IMPL>::f(x[0][i], x[1][i], x[2][i], alpha));
    }
    __syncthreads();                  // the tiles are rewritten by the next iteration
  }
}

// ---------------------------------------------------------------------------
// PATH_STAGED: contiguous [B, R, C] output (leading sizes may be 1: a matrix, a flat tensor), every
// input addressed by three strides of its own (any values, 0 on broadcast dims), any float dtype
// per operand, any alignment of the inputs: stride-2 slices, row and column vectors whatever C is,
// small transposes, operands of another dtype.  A round is 1024 consecutive output elements, four
// per lane.  For each input the workgroup first brings the contiguous span of memory that the
// round touches into LDS with coalesced 16-byte loads (every line is fetched once, whatever the
// stride), then each lane gathers its elements from LDS; the results leave as whole vectors.  An
// input whose span does not fit what is left of the LDS is read element by element for that
// round instead.
// ---------------------------------------------------------------------------
constexpr uint32_t kStageRound = 4u * kThreads;
constexpr int kStageLoads = 4;             // 16-byte loads per lane and input in flight while a window is staged

struct StagedCtx {     // what every round of a chunk shares (workgroup-uniform)
  const char* p[3];
  uint32_t dt[3], es[3], sb[3], sr[3], sc[3];
  uint32_t m_f32[3], m_f16[3], m_bf16[3];  // all ones for the input's dtype
  uint32_t R, C, RC, odt, oes, begin;
  char* po;
  rsrc_t ro;                               // the output rebased to the chunk: stores past it are dropped
  float alpha;
  char* lds;
};
template <int IMPL> DEV void staged_ctx(StagedCtx& c, const Record* r, uint32_t begin, uint32_t end, char* lds) {
  constexpr int N = Op<IMPL>::N;
  c.R = uni(r->size[1]); c.C = uni(r->size[2]); c.RC = c.R * c.C;
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    const int kk = k < N ? k : 0;
    c.p[k] = uni_ptr(r->ptr[kk]);
    c.dt[k] = uni(r->dtype[kk]);
    c.es[k] = c.dt[k] == GPUOS_F32 ? 4u : 2u;
    c.sb[k] = uni(r->stride[kk][0]); c.sr[k] = uni(r->stride[kk][1]); c.sc[k] = uni(r->stride[kk][2]);
    c.m_f32[k] = c.dt[k] == GPUOS_F32 ? ~0u : 0u;
    c.m_f16[k] = c.dt[k] == GPUOS_F16 ? ~0u : 0u;
    c.m_bf16[k] = c.dt[k] == GPUOS_BF16 ? ~0u : 0u;
  }
  c.odt = uni(r->dtype[3]);
  c.oes = c.odt == GPUOS_F32 ? 4u : 2u;
  c.po = (char*)uni_ptr(r->ptr[3]);
  c.ro = make_rsrc(c.po + (uint64_t)begin * c.oes, (end - begin) * c.oes);
  c.alpha = r->alpha;
  c.begin = begin;
  c.lds = lds;
}

// One round's gather, arithmetic and store: the elements [c0, c1) of the output, inputs staged at
// g_region (element g_lo of input k lies at byte g_region[k] of the LDS scratch).  FULL: the round
// has all its 1,024 elements (every lane four live ones, one whole-vector store).  ALL_STAGED:
// every input is in LDS, and the round holds no memory load at all.
template <int POL, int IMPL, bool FULL, bool ALL_STAGED>
DEV void staged_round(const StagedCtx& c, uint32_t c0, uint32_t c1, const uint32_t (&g_lo)[3], const uint32_t (&g_region)[3],
                      const bool (&g_staged)[3]) {
  using M = Mem<POL>;
  constexpr int N = Op<IMPL>::N;
  const uint32_t i = c0 + 4u * threadIdx.x;
  if (!FULL && i >= c1) return;
  uint32_t b = i / c.RC;
  const uint32_t j = i - b * c.RC;
  uint32_t row = j / c.C, col = j - row * c.C;
  float x[3][4], o[4];
  // the four elements' offsets first, then every read of a staged input in one go (one LDS latency
  // per input, not one per element): the aligned word that holds the element is read whatever the
  // dtype and the element is cut out of it afterwards
  uint32_t off[3][4];
  bool live[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    live[e] = FULL || i + e < c1;
#pragma unroll
    for (int k = 0; k < N; ++k) off[k][e] = b * c.sb[k] + row * c.sr[k] + col * c.sc[k];
    if (++col == c.C) { col = 0; if (++row == c.R) { row = 0; ++b; } }
  }
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    if (k >= N) {
#pragma unroll
      for (int e = 0; e < 4; ++e) x[k][e] = 0.0f;
    } else if (ALL_STAGED || g_staged[k]) {
      uint32_t w[4], at_byte[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        at_byte[e] = live[e] ? g_region[k] + (off[k][e] - g_lo[k]) * c.es[k] : g_region[k];
        w[e] = *(const uint32_t*)(c.lds + (at_byte[e] & ~3u));
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        // (masks, not branches on the dtype: the three decodings are a handful of operations)
        const uint32_t h = (at_byte[e] & 2u) ? (w[e] >> 16) : (w[e] & 0xffffu);
        const uint32_t bits = (w[e] & c.m_f32[k]) | (__builtin_bit_cast(uint32_t, h2f(h)) & c.m_f16[k]) | ((h << 16) & c.m_bf16[k]);
        x[k][e] = live[e] ? __builtin_bit_cast(float, bits) : 0.0f;
      }
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) x[k][e] = live[e] ? load_rt<POL>(c.p[k], off[k][e], c.dt[k]) : 0.0f;
    }
  }
  apply_vec<IMPL, 4>(x[0], x[1], x[2], c.alpha, o);
  const uint32_t rel = (i - c.begin) * c.oes;
  if (FULL) {
    // Both forms of the store are issued, the one that does not apply past the end of the window
    // (dropped, no traffic): the number of stores a wavefront has in flight after a full round is
    // then the same on every path, and the wait for the next round's vectors can leave them there.
    v4i qo;
#pragma unroll
    for (int e = 0; e < 4; ++e) qo[e] = __builtin_bit_cast(int, o[e]);
    uint32_t w0, w1;
    if (c.odt == GPUOS_F16) { w0 = f2h(o[0]) | (f2h(o[1]) << 16); w1 = f2h(o[2]) | (f2h(o[3]) << 16); }
    else { w0 = f2b(o[0]) | (f2b(o[1]) << 16); w1 = f2b(o[2]) | (f2b(o[3]) << 16); }
    M::st16(c.ro, c.odt == GPUOS_F32 ? rel : kNoLoad, qo);
    M::st8(c.ro, c.odt == GPUOS_F32 ? kNoLoad : rel, w0, w1);
  } else if (i + 4u <= c1) {
    if (c.odt == GPUOS_F32) {
      v4i qo;
#pragma unroll
      for (int e = 0; e < 4; ++e) qo[e] = __builtin_bit_cast(int, o[e]);
      M::st16(c.ro, rel, qo);
    } else {
      uint32_t w0, w1;
      if (c.odt == GPUOS_F16) { w0 = f2h(o[0]) | (f2h(o[1]) << 16); w1 = f2h(o[2]) | (f2h(o[3]) << 16); }
      else { w0 = f2b(o[0]) | (f2b(o[1]) << 16); w1 = f2b(o[2]) | (f2b(o[3]) << 16); }
      M::st8(c.ro, rel, w0, w1);
    }
  } else {
    for (uint32_t e = 0; i + e < c1; ++e) store_rt<POL>(c.po, i + e, c.odt, o[e]);      // the chunk's ragged end
  }
}

// A round with an input whose window does not fit the LDS scratch (that input is read element by
// element): a function of its own, so that its memory loads and the waits for them stay out of the
// common round's code.
template <int POL, int IMPL>
PATHFN void ew_staged_slow_round(const Record* r_v, uint32_t begin_v, uint32_t end_v, float* s_v, uint32_t c0_v, uint32_t c1_v,
                                 uint32_t lo0, uint32_t lo1, uint32_t lo2, uint32_t rg0, uint32_t rg1, uint32_t rg2, uint32_t staged_mask_v) {
  const Record* r = lds_arg(r_v);
  StagedCtx c;
  staged_ctx<IMPL>(c, r, uni(begin_v), uni(end_v), (char*)lds_arg(s_v));
  const uint32_t g_lo[3] = {uni(lo0), uni(lo1), uni(lo2)}, g_region[3] = {uni(rg0), uni(rg1), uni(rg2)};
  const uint32_t mask = uni(staged_mask_v);
  const bool g_staged[3] = {(mask & 1u) != 0, (mask & 2u) != 0, (mask & 4u) != 0};
  staged_round<POL, IMPL, false, false>(c, uni(c0_v), uni(c1_v), g_lo, g_region, g_staged);
}

template <int POL, int IMPL>
PATHFN void ew_staged(const Record* r_v, uint32_t begin_v, uint32_t end_v, float* s_v) {
  const Record* r = lds_arg(r_v);
  const uint32_t begin = uni(begin_v), end = uni(end_v);
  char* lds = (char*)lds_arg(s_v);
  using M = Mem<POL>;
  constexpr int N = Op<IMPL>::N;
  StagedCtx c;
  staged_ctx<IMPL>(c, r, begin, end, lds);
  const uint32_t tid = threadIdx.x;
  constexpr uint32_t kLdsBytes = kScratchFloats * 4u;
  constexpr uint32_t kBatchBytes = kStageLoads * kThreads * 16u;
  static_assert(kStageLoads == 4, "the pin in stash() names four vectors");
  // What a round stages (uniform): for every input the 16-byte window of memory its elements lie in.
  uint32_t lo[3] = {0, 0, 0}, region[3] = {0, 0, 0}, at[3], nbs[3], most = 0;
  bool staged[3] = {true, true, true};
  rsrc_t rs[3];
  auto plan = [&](uint32_t i0, uint32_t i1) {
    // indices of the first and the last element of the round
    const uint32_t ba = i0 / c.RC, ja = i0 - ba * c.RC, ra = ja / c.C, ca = ja - ra * c.C;
    const uint32_t bb = (i1 - 1) / c.RC, jb = (i1 - 1) - bb * c.RC, rb = jb / c.C, cb = jb - rb * c.C;
    uint32_t used = 0;
    most = 0;
#pragma unroll
    for (int k = 0; k < N; ++k) {
      // bounds on the element offsets the round can touch (strides are non-negative): exact up to
      // the outermost index in which its first and last element differ, everything inside that
      uint32_t first, last;
      if (ba != bb) { first = ba * c.sb[k]; last = bb * c.sb[k] + (c.R - 1u) * c.sr[k] + (c.C - 1u) * c.sc[k]; }
      else if (ra != rb) { first = ba * c.sb[k] + ra * c.sr[k]; last = ba * c.sb[k] + rb * c.sr[k] + (c.C - 1u) * c.sc[k]; }
      else { first = ba * c.sb[k] + ra * c.sr[k] + ca * c.sc[k]; last = ba * c.sb[k] + ra * c.sr[k] + cb * c.sc[k]; }
      // the window in whole 16-byte vectors of the address space (the base need not be aligned)
      const uint64_t a_first = (uint64_t)(__UINTPTR_TYPE__)c.p[k] + (uint64_t)first * c.es[k];
      const uint64_t a_last = (uint64_t)(__UINTPTR_TYPE__)c.p[k] + (uint64_t)last * c.es[k] + c.es[k];
      const uint64_t v_first = a_first & ~15ull;
      const uint64_t bytes = ((a_last + 15ull) & ~15ull) - v_first;
      staged[k] = bytes <= (uint64_t)(kLdsBytes - used);
      lo[k] = first;
      // an input that is not staged gets an empty window: its loads fetch nothing
      nbs[k] = staged[k] ? (uint32_t)bytes : 0u;
      rs[k] = make_rsrc((const void*)(__UINTPTR_TYPE__)v_first, nbs[k]);
      at[k] = used;
      region[k] = used + (uint32_t)(a_first - v_first);            // where element `first` lies inside the staged bytes
      used += nbs[k];
      most = nbs[k] > most ? nbs[k] : most;
    }
  };
  // The windows of all inputs move together, kStageLoads vectors per lane and input in flight: every
  // load of a batch is issued before the first one is written to LDS (one memory latency per batch,
  // not one per vector and input).  Loads past a window's end are dropped by its bounds check.
  v4i q[N][kStageLoads];
  auto issue = [&](uint32_t b0) {
#pragma unroll
    for (int k = 0; k < N; ++k)
#pragma unroll
      for (int u = 0; u < kStageLoads; ++u) q[k][u] = M::ld16(rs[k], b0 + (tid + u * kThreads) * 16u);
  };
  auto stash = [&](uint32_t b0) {
    // (the values are pinned here: a load used only under the condition below would be moved there,
    // behind the waits of the stores before it)
#pragma unroll
    for (int k = 0; k < N; ++k) asm volatile("" : "+v"(q[k][0]), "+v"(q[k][1]), "+v"(q[k][2]), "+v"(q[k][3]));
#pragma unroll
    for (int k = 0; k < N; ++k)
#pragma unroll
      for (int u = 0; u < kStageLoads; ++u) {
        const uint32_t off = b0 + (tid + u * kThreads) * 16u;
        if (off < nbs[k]) *(v4i*)(lds + at[k] + off) = q[k][u];
      }
  };
  // Rounds are pipelined: the first batch of the NEXT round's windows is requested before this
  // round's elements are gathered and computed, so from the second round on the memory latency
  // hides behind the round before.  A round that has a successor is a full one, and every
  // wavefront issues exactly one store in it after those requests: the wait for the requested
  // vectors can leave that one store in flight.
  uint32_t i0 = begin, i1 = (end - begin < kStageRound) ? end : begin + kStageRound;
  plan(i0, i1);
  issue(0);
  stash(0);
  for (uint32_t b0 = kBatchBytes; b0 < most; b0 += kBatchBytes) { issue(b0); stash(b0); }
  __syncthreads();
  uint32_t c0, c1, g_lo[3], g_region[3];
  bool g_staged[3], all_staged;
  auto take = [&]() {                 // this round's share of the plan; the plan itself moves on
    c0 = i0; c1 = i1;
    all_staged = true;
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      g_lo[k] = lo[k]; g_region[k] = region[k]; g_staged[k] = staged[k];
      if (k < N) all_staged = all_staged && staged[k];
    }
  };
  auto slow_round = [&]() {
    const uint32_t mask = (g_staged[0] ? 1u : 0u) | (g_staged[1] ? 2u : 0u) | (g_staged[2] ? 4u : 0u);
    ew_staged_slow_round<POL, IMPL>(r_v, begin, end, s_v, c0, c1, g_lo[0], g_lo[1], g_lo[2], g_region[0], g_region[1], g_region[2], mask);
  };
  while (i1 < end) {                  // a round with a successor
    take();
    if (!all_staged) break;           // (rare) the rest of the chunk goes round by round below
    i0 = c1;
    i1 = (end - i0 < kStageRound) ? end : i0 + kStageRound;
    plan(i0, i1);
    issue(0);
    staged_round<POL, IMPL, true, true>(c, c0, c1, g_lo, g_region, g_staged);
    __syncthreads();                  // the staged windows may be overwritten now
    stash(0);
    for (uint32_t b0 = kBatchBytes; b0 < most; b0 += kBatchBytes) { issue(b0); stash(b0); }
    __syncthreads();
  }
  // The chunk's last round, and every round from the first one on that has an input too wide to
  // stage: one after the other.
  for (;;) {
    take();
    if (all_staged) staged_round<POL, IMPL, false, true>(c, c0, c1, g_lo, g_region, g_staged);
    else slow_round();
    __syncthreads();                  // the scratch may be reused (by the next round, by the next chunk)
    if (i1 >= end) break;
    i0 = c1;
    i1 = (end - i0 < kStageRound) ? end : i0 + kStageRound;
    plan(i0, i1);
    issue(0);
    stash(0);
    for (uint32_t b0 = kBatchBytes; b0 < most; b0 += kBatchBytes) { issue(b0); stash(b0); }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------
// PATH_GENERIC: row-major index decomposition over <= 6 coalesced dims, per
// operand strides (0 on broadcast dims), per operand dtype.
// ---------------------------------------------------------------------------
template <int POL, int IMPL, bool INT>
PATHFN void ew_generic(const Record* r_v, uint32_t begin_v, uint32_t end_v) {
  const Record* r = lds_arg(r_v);
  const uint32_t begin = uni(begin_v), end = uni(end_v);
  using M = Mem<POL>;
  constexpr int N = INT ? 2 : Op<IMPL>::N;
  const int nd = (int)uni(r->ndim);
  const int nin = (int)uni(r->n_inputs);
  uint32_t size[GPUOS_MAX_DIMS], st[4][GPUOS_MAX_DIMS];
#pragma unroll
  for (int d = 0; d < GPUOS_MAX_DIMS; ++d) {
    size[d] = uni(r->size[d]);
#pragma unroll
    for (int k = 0; k < 4; ++k) st[k][d] = uni(r->stride[k][d]);
  }
  const char* p[3];
  uint32_t dt[4];
#pragma unroll
  for (int k = 0; k < 3; ++k) { p[k] = uni_ptr(r->ptr[k]); dt[k] = uni(r->dtype[k]); }
  dt[3] = uni(r->dtype[3]);
  char* po = (char*)uni_ptr(r->ptr[3]);
  const float alpha = r->alpha;
  for (uint32_t i = begin + threadIdx.x; i < end; i += kThreads) {
    uint32_t rem = i, off[4] = {0, 0, 0, 0};
#pragma unroll
    for (int d = GPUOS_MAX_DIMS - 1; d >= 0; --d) {
      if (d < nd) {
        const uint32_t q = rem / size[d];
        const uint32_t idx = rem - q * size[d];
        rem = q;
#pragma unroll
        for (int k = 0; k < 4; ++k) off[k] += idx * st[k][d];
      }
    }
    if (INT) {
      const uint32_t x = M::ld4(p[0], off[0]);
      const uint32_t y = nin > 1 ? M::ld4(p[1], off[1]) : 0u;
      M::st4(po, off[3], int_op<IMPL>(x, y));
    } else if (IMPL == GPUOS_IMPL_COPY && dt[0] == dt[3]) {
      if (dt[0] == GPUOS_F32) M::st4(po, off[3], M::ld4(p[0], off[0]));
      else M::st2(po, off[3], M::ld2(p[0], off[0]));
    } else {
      const float x = load_rt<POL>(p[0], off[0], dt[0]);
      const float y = N > 1 ? load_rt<POL>(p[1], off[1], dt[1]) : 0.f;
      const float z = N > 2 ? load_rt<POL>(p[2], off[2], dt[2]) : 0.f;
      store_rt<POL>(po, off[3], dt[3], Op<IMPL>::f(x, y, z, alpha));
    }
  }
}

// ---------------------------------------------------------------------------
// reductions over the last dim
// ---------------------------------------------------------------------------
template <int RIMPL> DEV float red_identity() {
  return RIMPL == GPUOS_IMPL_SUM_LAST ? 0.0f : (RIMPL == GPUOS_IMPL_MAX_LAST ? -__builtin_inff() : __builtin_inff());
}
template <int RIMPL> DEV float red_combine(float a, float b) {
  if (RIMPL == GPUOS_IMPL_SUM_LAST) return a + b;
  if (a != a) return a;                               // max / min propagate NaN
  if (b != b) return b;
  if (RIMPL == GPUOS_IMPL_MAX_LAST) return a > b ? a : b;
  return a < b ? a : b;
}
template <int RIMPL> DEV int32_t red_identity_i() {
  return RIMPL == GPUOS_IMPL_SUM_LAST ? 0 : (RIMPL == GPUOS_IMPL_MAX_LAST ? (int32_t)0x80000000 : 0x7fffffff);
}
template <int RIMPL> DEV int32_t red_combine_i(int32_t a, int32_t b) {
  if (RIMPL == GPUOS_IMPL_SUM_LAST) return (int32_t)((uint32_t)a + (uint32_t)b);
  if (RIMPL == GPUOS_IMPL_MAX_LAST) return a > b ? a : b;
  return a < b ? a : b;
}

// The partner of a lane in step OFF of an all-reduce butterfly over aligned groups of 2 * OFF
// lanes.  Steps 1 and 2 swap inside a quad and steps 4 and 8 mirror a half row / a row of 16 lanes
// (lane i with i ^ 7, i ^ 15): DPP operand modifiers, no trip through the LDS crossbar that a
// shuffle takes.  The masks 1, 2, 7, 15, 16, 32 are independent, so the steps still reach every
// lane of the group.  Steps 16 and 32 cross rows and stay shuffles.  All lanes must be active.
template <int OFF> DEV int butterfly_partner(int v) {
  if (OFF == 1) return __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xf, 0xf, false);      // quad_perm [1,0,3,2]
  if (OFF == 2) return __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xf, 0xf, false);      // quad_perm [2,3,0,1]
  if (OFF == 4) return __builtin_amdgcn_update_dpp(v, v, 0x141, 0xf, 0xf, false);     // row_half_mirror
  if (OFF == 8) return __builtin_amdgcn_update_dpp(v, v, 0x140, 0xf, 0xf, false);     // row_mirror
  return __shfl_xor(v, OFF, 64);
}
template <int OFF> DEV float butterfly_partner(float v) {
  return __builtin_bit_cast(float, butterfly_partner<OFF>(__builtin_bit_cast(int, v)));
}

// all-reduce over the `width` lanes (power of two <= 64, aligned) a lane belongs to
template <int RIMPL> DEV float wave_reduce(float acc, uint32_t width) {
  if (width > 32) acc = red_combine<RIMPL>(acc, butterfly_partner<32>(acc));
  if (width > 16) acc = red_combine<RIMPL>(acc, butterfly_partner<16>(acc));
  if (width > 8) acc = red_combine<RIMPL>(acc, butterfly_partner<8>(acc));
  if (width > 4) acc = red_combine<RIMPL>(acc, butterfly_partner<4>(acc));
  if (width > 2) acc = red_combine<RIMPL>(acc, butterfly_partner<2>(acc));
  if (width > 1) acc = red_combine<RIMPL>(acc, butterfly_partner<1>(acc));
  return acc;
}
template <int RIMPL> DEV int32_t wave_reduce_i(int32_t acc, uint32_t width) {
  if (width > 32) acc = red_combine_i<RIMPL>(acc, butterfly_partner<32>(acc));
  if (width > 16) acc = red_combine_i<RIMPL>(acc, butterfly_partner<16>(acc));
  if (width > 8) acc = red_combine_i<RIMPL>(acc, butterfly_partner<8>(acc));
  if (width > 4) acc = red_combine_i<RIMPL>(acc, butterfly_partner<4>(acc));
  if (width > 2) acc = red_combine_i<RIMPL>(acc, butterfly_partner<2>(acc));
  if (width > 1) acc = red_combine_i<RIMPL>(acc, butterfly_partner<1>(acc));
  return acc;
}

// PATH_RED_CONTIG: input is a contiguous [rows, n] matrix of dtype DT, output a
// contiguous vector [rows] of any float dtype.  The rows of a chunk are read as one flat
// run of 16-byte vectors aligned to the tensor base, whatever n is: a vector that straddles
// a row boundary is loaded by both rows and masked per element.  Three shapes of work:
//   short rows  (span <= 64 vectors): P lanes per row, 64 / P rows per wavefront pass,
//               four passes in flight;
//   medium rows: one wavefront per row, RA rows at a time, UN loads per row in flight;
//   long rows   (>= 1024 vectors): the four wavefronts take a quarter of each row, partial
//               results meet in LDS once per chunk (one barrier per chunk, not per row).
// Per-element accumulation.  SUM adds.  MAX / MIN must propagate NaN: the running value ignores
// NaN (one compare + select) and `nan` remembers whether one was seen (one unordered compare,
// or-ed into a wavefront-uniform mask register); red_finish folds the two before the lanes are combined.
template <int RIMPL> DEV float red_step(float acc, float x, bool& nan) {
  if (RIMPL == GPUOS_IMPL_SUM_LAST) return acc + x;
  nan = nan || (x != x);
  if (RIMPL == GPUOS_IMPL_MAX_LAST) return x > acc ? x : acc;
  return x < acc ? x : acc;
}
template <int RIMPL> DEV float red_finish(float acc, bool nan) {
  if (RIMPL == GPUOS_IMPL_SUM_LAST) return acc;
  return nan ? __builtin_nanf("") : acc;
}

// Two elements per step for max / min: one three-operand max (min) and ONE unordered compare of
// the two new elements with each other, which is true exactly when either is a NaN.  The hardware
// max / min skip quiet NaNs, which is fine: the flag decides the result (red_finish).  Three
// operations per element (compare, compare, select) become one; the 16-bit reductions were
// bound by them.
template <int RIMPL> DEV float red_step2(float acc, float x0, float x1, bool& nan) {
  nan = nan || __builtin_isunordered(x0, x1);
  float r;
  if (RIMPL == GPUOS_IMPL_MAX_LAST) asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(acc), "v"(x0), "v"(x1));
  else asm("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(acc), "v"(x0), "v"(x1));
  return r;
}

template <int RIMPL, int DT>
DEV float red_vector(const v4i& q, uint32_t f0, uint32_t lo, uint32_t hi, bool edge, float acc, bool& nan) {
  // q holds elements f0 .. f0+V-1 of the flat run; the row is [lo, hi)
  using E = Elem<DT>;
  if (!edge) {
    if (RIMPL == GPUOS_IMPL_SUM_LAST) {
#pragma unroll
      for (int k = 0; k < E::V; ++k) acc = red_step<RIMPL>(acc, E::get(q, k), nan);
    } else {
#pragma unroll
      for (int k = 0; k < E::V; k += 2) acc = red_step2<RIMPL>(acc, E::get(q, k), E::get(q, k + 1), nan);
    }
  } else {
#pragma unroll
    for (int k = 0; k < E::V; ++k)
      if (f0 + k >= lo && f0 + k < hi) acc = red_step<RIMPL>(acc, E::get(q, k), nan);
  }
  return acc;
}


struct RedArgs {       // what a row-reduction variant is called with (plain values: see lds_arg)
  const char* base;    // first byte of the run: the tensor base advanced to the chunk's first vector
  uint32_t bytes;      // length of the run, whole vectors
  uint32_t base_elem;  // first element of the run (multiple of V), relative to the tensor
  uint32_t n;
  char* po;
  uint32_t odt, row_begin, row_end, max_span;
  float* s_part;       // LDS
};
struct RedRun {        // the chunk's rows as a flat run of vectors
  rsrc_t rin;
  uint32_t base_elem;
  uint32_t n;
};
DEV RedRun red_run(const RedArgs& a) {
  RedRun run;
  run.rin = make_rsrc(uni_ptr((uint64_t)a.base), uni(a.bytes));
  run.base_elem = uni(a.base_elem);
  run.n = uni(a.n);
  return run;
}

template <int POL, int RIMPL, int DT, int RA, int UN>
PATHFN void red_rows_wave(RedArgs a) {
  const RedRun run = red_run(a);
  char* po = (char*)uni_ptr((uint64_t)a.po);
  const uint32_t odt = uni(a.odt), row_begin = uni(a.row_begin), row_end = uni(a.row_end);
  using E = Elem<DT>;
  using M = Mem<POL>;
  constexpr uint32_t V = E::V;
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  const uint32_t n = run.n;
  // wave w takes rows row_begin + w, + 4, + 8, ... ; RA of them at a time
  for (uint32_t row0 = row_begin + wave; row0 < row_end; row0 += 4 * RA) {
    float acc[RA];
    bool nan[RA];
    uint32_t lo[RA], hi[RA], j0[RA], j1[RA];
    uint32_t span = 0;
#pragma unroll
    for (int i = 0; i < RA; ++i) {
      acc[i] = red_identity<RIMPL>();
      nan[i] = false;
      const uint32_t row = row0 + 4 * i;
      lo[i] = row * n - run.base_elem;
      hi[i] = lo[i] + n;
      j0[i] = lo[i] / V;
      j1[i] = (hi[i] - 1) / V;
      if (row >= row_end) { hi[i] = lo[i]; j1[i] = j0[i]; }
      const uint32_t sp = j1[i] - j0[i] + 1;
      span = sp > span ? sp : span;
    }
    for (uint32_t v = lane; v < span; v += 64 * UN) {
      v4i q[RA][UN];
#pragma unroll
      for (int i = 0; i < RA; ++i)
#pragma unroll
        for (int u = 0; u < UN; ++u) {   // vectors past the row are not fetched
          const uint32_t j = j0[i] + v + u * 64;
          q[i][u] = M::ld16(run.rin, (j <= j1[i] && hi[i] > lo[i]) ? j * 16u : kNoLoad);
        }
#pragma unroll
      for (int i = 0; i < RA; ++i)
#pragma unroll
        for (int u = 0; u < UN; ++u) {
          const uint32_t j = j0[i] + v + u * 64;
          if (j <= j1[i] && hi[i] > lo[i])
            acc[i] = red_vector<RIMPL, DT>(q[i][u], j * V, lo[i], hi[i], j == j0[i] || j == j1[i], acc[i], nan[i]);
        }
    }
#pragma unroll
    for (int i = 0; i < RA; ++i) {
      const float t = wave_reduce<RIMPL>(red_finish<RIMPL>(acc[i], nan[i]), 64);
      if (lane == 0 && row0 + 4 * i < row_end) store_rt<POL>(po, row0 + 4 * i, odt, t);
    }
  }
}

constexpr uint32_t kRedPartialRows = 64;   // rows of partial results the LDS scratch holds

template <int POL, int RIMPL, int DT>
PATHFN void red_rows_quarter(RedArgs a) {
  const RedRun run = red_run(a);
  char* po = (char*)uni_ptr((uint64_t)a.po);
  const uint32_t odt = uni(a.odt), row_begin = uni(a.row_begin), row_end = uni(a.row_end);
  float* s_part = lds_arg(a.s_part);
  using E = Elem<DT>;
  using M = Mem<POL>;
  constexpr uint32_t V = E::V;
  constexpr int UN = 8;
  const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  const uint32_t n = run.n;
  for (uint32_t row = row_begin; row < row_end; ++row) {
    const uint32_t lo = row * n - run.base_elem, hi = lo + n;
    const uint32_t j0 = lo / V, j1 = (hi - 1) / V;
    const uint32_t span = j1 - j0 + 1, sq = (span + 3u) / 4u;          // vectors per quarter
    const uint32_t q_begin = j0 + wave * sq;
    const uint32_t q_end = (q_begin + sq <= j1 + 1) ? q_begin + sq : j1 + 1;
    float a0 = red_identity<RIMPL>(), a1 = a0;
    bool nan = false;
    for (uint32_t v = q_begin + lane; v < q_end; v += 64 * UN) {
      v4i q[UN];
#pragma unroll
      for (int u = 0; u < UN; ++u) q[u] = M::ld16(run.rin, (v + u * 64 < q_end) ? (v + u * 64) * 16u : kNoLoad);
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        const uint32_t j = v + u * 64;
        if (j < q_end) {
          if ((u & 1) == 0) a0 = red_vector<RIMPL, DT>(q[u], j * V, lo, hi, j == j0 || j == j1, a0, nan);
          else a1 = red_vector<RIMPL, DT>(q[u], j * V, lo, hi, j == j0 || j == j1, a1, nan);
        }
      }
    }
    const float t = wave_reduce<RIMPL>(red_finish<RIMPL>(red_combine<RIMPL>(a0, a1), nan), 64);
    if (lane == 0) s_part[(row - row_begin) * 4 + wave] = t;
  }
  __syncthreads();
  const uint32_t nrows = row_end - row_begin;
  if (tid < nrows) {
    const float* p = s_part + tid * 4;
    const float t = red_combine<RIMPL>(red_combine<RIMPL>(p[0], p[1]), red_combine<RIMPL>(p[2], p[3]));
    store_rt<POL>(po, row_begin + tid, odt, t);
  }
  __syncthreads();
}

template <int POL, int RIMPL, int DT>
PATHFN void red_rows_short(RedArgs a) {
  const RedRun run = red_run(a);
  char* po = (char*)uni_ptr((uint64_t)a.po);
  const uint32_t odt = uni(a.odt), row_begin = uni(a.row_begin), row_end = uni(a.row_end), max_span = uni(a.max_span);
  using E = Elem<DT>;
  using M = Mem<POL>;
  constexpr uint32_t V = E::V;
  constexpr int UP = 8;
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  const uint32_t n = run.n;
  uint32_t P = 1;                                     // lanes per row: power of two >= the widest span
  while (P < max_span) P <<= 1;
  const uint32_t rpw = 64u / P, sub = lane / P, j = lane & (P - 1u);
  const bool gather = UP * rpw <= 64u;                // the pass's rows fit one lane each
  // one wavefront pass covers the UP * rpw consecutive rows base .. base + UP * rpw - 1
  for (uint32_t base = row_begin + wave * rpw * UP; base < row_end; base += 4 * rpw * UP) {
    v4i q[UP];
    uint32_t lo[UP], hi[UP], j0[UP], j1[UP];
#pragma unroll
    for (int u = 0; u < UP; ++u) {
      const uint32_t row = base + u * rpw + sub;
      lo[u] = row * n - run.base_elem;
      hi[u] = lo[u] + n;
      j0[u] = lo[u] / V;
      j1[u] = (hi[u] - 1) / V;
      q[u] = M::ld16(run.rin, (row < row_end && j0[u] + j <= j1[u]) ? (j0[u] + j) * 16u : kNoLoad);
    }
    float mine = 0.0f;                                // lane L ends up with the result of row base + L
#pragma unroll
    for (int u = 0; u < UP; ++u) {
      const uint32_t row = base + u * rpw + sub;
      const uint32_t jj = j0[u] + j;
      float acc = red_identity<RIMPL>();
      bool nan = false;
      if (row < row_end && jj <= j1[u])
        acc = red_vector<RIMPL, DT>(q[u], jj * V, lo[u], hi[u], jj == j0[u] || jj == j1[u], acc, nan);
      acc = wave_reduce<RIMPL>(red_finish<RIMPL>(acc, nan), P);
      // every lane of sub-group s now holds the result of row base + u * rpw + s
      if (gather) {
        const float got = __shfl(acc, (int)((lane & (rpw - 1u)) * P), 64);
        if (lane / rpw == (uint32_t)u) mine = got;
      } else if (row < row_end && j == 0) {
        store_rt<POL>(po, row, odt, acc);            // rows of one or two vectors: the owners are adjacent lanes already
      }
    }
    // UP * rpw consecutive rows, one lane each: a coalesced store instead of one 4-byte store per row
    if (gather && lane < UP * rpw && base + lane < row_end) store_rt<POL>(po, base + lane, odt, mine);
  }
}

// The same when every row is a whole number of vectors and starts on one (the attention shapes: rows
// of 64 / 128 / 256 16-bit elements): no edges to mask and nothing to remember per pass but the
// loaded vector, so eight passes stay in registers.
template <int POL, int RIMPL, int DT>
PATHFN void red_rows_short_aligned(RedArgs a) {
  const RedRun run = red_run(a);
  char* po = (char*)uni_ptr((uint64_t)a.po);
  const uint32_t odt = uni(a.odt), row_begin = uni(a.row_begin), row_end = uni(a.row_end), vpr = uni(a.max_span);
  using M = Mem<POL>;
  constexpr int UP = 8;
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  uint32_t P = 1;                                     // lanes per row: power of two >= vectors per row
  while (P < vpr) P <<= 1;
  const uint32_t rpw = 64u / P, sub = lane / P, j = lane & (P - 1u);
  const bool gather = UP * rpw <= 64u;                // the pass's rows fit one lane each
  const bool mine = j < vpr;
  for (uint32_t base = row_begin + wave * rpw * UP; base < row_end; base += 4 * rpw * UP) {
    v4i q[UP];
#pragma unroll
    for (int u = 0; u < UP; ++u) {
      const uint32_t row = base + u * rpw + sub;
      q[u] = M::ld16(run.rin, (row < row_end && mine) ? ((row - row_begin) * vpr + j) * 16u : kNoLoad);
    }
    float res = 0.0f;                                 // lane L ends up with the result of row base + L
#pragma unroll
    for (int u = 0; u < UP; ++u) {
      const uint32_t row = base + u * rpw + sub;
      float acc = red_identity<RIMPL>();
      bool nan = false;
      if (row < row_end && mine) acc = red_vector<RIMPL, DT>(q[u], 0, 0, 0, false, acc, nan);
      acc = wave_reduce<RIMPL>(red_finish<RIMPL>(acc, nan), P);
      if (gather) {
        const float got = __shfl(acc, (int)((lane & (rpw - 1u)) * P), 64);
        if (lane / rpw == (uint32_t)u) res = got;
      } else if (row < row_end && j == 0) {
        store_rt<POL>(po, row, odt, acc);
      }
    }
    if (gather && lane < UP * rpw && base + lane < row_end) store_rt<POL>(po, base + lane, odt, res);
  }
}

template <int POL, int RIMPL, int DT>
DEV void red_contig(const Record* r, uint32_t row_begin, uint32_t row_end, float* s_part) {
  using E = Elem<DT>;
  constexpr uint32_t V = E::V;
  const uint32_t n = uni(r->red_n);
  const char* pin = uni_ptr(r->ptr[0]);
  char* po = (char*)uni_ptr(r->ptr[3]);
  const uint32_t odt = uni(r->dtype[3]);
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  if (r->rflags & RF_VEC) {                           // tensor base is 16-byte aligned
    RedArgs a;
    a.n = n;
    a.base_elem = (row_begin * n) / V * V;            // chunk start, aligned down to a vector
    // end rounded up to a whole vector (the base is 16-byte aligned, so the padding stays inside
    // the 16-byte block that holds the last element); vector loads further out read zeros; both
    // are masked per element
    a.base = pin + (uint64_t)a.base_elem * E::ES;
    a.bytes = ((row_end * n - a.base_elem) * E::ES + 15u) & ~15u;
    a.po = po; a.odt = odt; a.row_begin = row_begin; a.row_end = row_end; a.s_part = s_part;
    a.max_span = (n % V == 0 && a.base_elem == row_begin * n) ? n / V : (n + V - 2) / V + 1;
    if (a.max_span <= 64u && n % V == 0 && a.base_elem == row_begin * n) red_rows_short_aligned<POL, RIMPL, DT>(a);
    else if (a.max_span <= 64u) red_rows_short<POL, RIMPL, DT>(a);
    else if (a.max_span >= 1024u && row_end - row_begin <= kRedPartialRows) red_rows_quarter<POL, RIMPL, DT>(a);
    else if (a.max_span < 256u) red_rows_wave<POL, RIMPL, DT, 4, 2>(a);
    else red_rows_wave<POL, RIMPL, DT, 2, 4>(a);
    return;
  }
  // tensor base not 16-byte aligned: one wave per row, element loads
  for (uint32_t row = row_begin + wave; row < row_end; row += 4) {
    const char* prow = pin + (uint64_t)row * n * E::ES;
    float acc = red_identity<RIMPL>();
    for (uint32_t jx = lane; jx < n; jx += 64) acc = red_combine<RIMPL>(acc, E::template load1<POL>(prow, jx));
    acc = wave_reduce<RIMPL>(acc, 64);
    if (lane == 0) store_rt<POL>(po, row, odt, acc);
  }
}

// PATH_RED_GENERIC: one wave per output row; outer index decomposed over the
// coalesced outer dims; stride[0][5] walks the reduced dim.
template <int POL, int RIMPL, bool INT>
PATHFN void red_generic(const Record* r_v, uint32_t begin_v, uint32_t end_v) {
  const Record* r = lds_arg(r_v);
  const uint32_t row_begin = uni(begin_v), row_end = uni(end_v);
  using M = Mem<POL>;
  const int nd = (int)uni(r->ndim);                   // outer dims
  const uint32_t n = uni(r->red_n), sl = uni(r->stride[0][5]);
  const char* pin = uni_ptr(r->ptr[0]);
  char* po = (char*)uni_ptr(r->ptr[3]);
  const uint32_t idt = uni(r->dtype[0]), odt = uni(r->dtype[3]);
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  for (uint32_t row = row_begin + wave; row < row_end; row += 4) {
    uint32_t rem = row, ioff = 0, ooff = 0;
#pragma unroll
    for (int d = GPUOS_MAX_DIMS - 2; d >= 0; --d) {
      if (d < nd) {
        const uint32_t sz = uni(r->size[d]);
        const uint32_t q = rem / sz, idx = rem - q * sz;
        rem = q;
        ioff += idx * uni(r->stride[0][d]);
        ooff += idx * uni(r->stride[3][d]);
      }
    }
    if (INT) {
      int32_t acc = red_identity_i<RIMPL>();
      for (uint32_t jx = lane; jx < n; jx += 64) acc = red_combine_i<RIMPL>(acc, (int32_t)M::ld4(pin, ioff + jx * sl));
      acc = wave_reduce_i<RIMPL>(acc, 64);
      if (lane == 0) M::st4(po, ooff, (uint32_t)acc);
    } else {
      float acc = red_identity<RIMPL>();
      for (uint32_t jx = lane; jx < n; jx += 64) acc = red_combine<RIMPL>(acc, load_rt<POL>(pin, ioff + jx * sl, idt));
      acc = wave_reduce<RIMPL>(acc, 64);
      if (lane == 0) store_rt<POL>(po, ooff, odt, acc);
    }
  }
}

// ---------------------------------------------------------------------------
// fused row operations (operator library, Section 5.2: softmax, layer normalisation).
// Each row of the last dim is one problem; the output has the input's shape.
//   PATH_ROW_FUSED: one dtype, contiguous rows of whole aligned 16-byte vectors, at most 256
//     vectors per row.  A row is read once into the registers of the P lanes that own it
//     (P = 64 for rows over 64 vectors, else the power of two >= vectors per row, 64 / P rows
//     per wavefront pass), reduced with xor butterflies over those lanes, and written once.
//   PATH_ROW_GENERIC: any strides and dtypes; one wavefront per row, three passes over memory.
// Arithmetic is fp32.  Lanes outside a row feed the identity (-inf to the softmax, 0 to the
// sums).  The softmax maximum ignores NaN; a NaN still poisons its row through the sum.
// ---------------------------------------------------------------------------
DEV float bfly_sum(float v, uint32_t width) {
  if (width > 32) v += butterfly_partner<32>(v);
  if (width > 16) v += butterfly_partner<16>(v);
  if (width > 8) v += butterfly_partner<8>(v);
  if (width > 4) v += butterfly_partner<4>(v);
  if (width > 2) v += butterfly_partner<2>(v);
  if (width > 1) v += butterfly_partner<1>(v);
  return v;
}
DEV float bfly_max(float v, uint32_t width) {
  if (width > 32) v = __builtin_fmaxf(v, butterfly_partner<32>(v));
  if (width > 16) v = __builtin_fmaxf(v, butterfly_partner<16>(v));
  if (width > 8) v = __builtin_fmaxf(v, butterfly_partner<8>(v));
  if (width > 4) v = __builtin_fmaxf(v, butterfly_partner<4>(v));
  if (width > 2) v = __builtin_fmaxf(v, butterfly_partner<2>(v));
  if (width > 1) v = __builtin_fmaxf(v, butterfly_partner<1>(v));
  return v;
}

template <int ROP> struct RowOp {
  static constexpr int NIN = ROP == GPUOS_IMPL_SOFTMAX_LAST ? 1 : (ROP == GPUOS_IMPL_MASKED_SOFTMAX_LAST ? 2 : 3);
  static constexpr bool SOFTMAX = ROP != GPUOS_IMPL_LAYERNORM_LAST;
};

// gamma / beta of a layer norm for the V elements of one vector position: of x's dtype (one
// 16-byte vector), or fp32 under 16-bit x (P32: two vectors), as frameworks keep them.
template <int POL, int DT, bool P32> struct RowParam {
  v4i q[P32 ? 2 : 1];
  DEV void load(rsrc_t rs, uint32_t vec) {
    if (P32) { q[0] = Mem<POL>::ld16(rs, vec * 32u); q[P32 ? 1 : 0] = Mem<POL>::ld16(rs, vec * 32u + 16u); }
    else q[0] = Mem<POL>::ld16(rs, vec * 16u);
  }
  DEV float get(int e) const {
    if (P32) return Elem<GPUOS_F32>::get(q[(e >> 2) & (P32 ? 1 : 0)], e & 3);
    return Elem<DT>::get(q[0], e);
  }
};

template <int POL, int ROP, int DT, int KW, int UP, bool P32 = false>
DEV void rowop_fused(const Record* r, uint32_t row_begin, uint32_t row_end) {
  using E = Elem<DT>;
  using M = Mem<POL>;
  using RO = RowOp<ROP>;
  constexpr uint32_t V = E::V;
  const uint32_t n = uni(r->red_n), vpr = n / V;
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  uint32_t P = 64;
  if (KW == 1) { P = 1; while (P < vpr) P <<= 1; }
  const uint32_t rpw = 64u / P, sub = lane / P, j = lane & (P - 1u);
  const float alpha = r->alpha;
  const uint32_t nrows = row_end - row_begin;
  const uint32_t chunk_bytes = nrows * n * E::ES;
  const uint64_t chunk_off = (uint64_t)row_begin * n * E::ES;
  const rsrc_t rx = make_rsrc(uni_ptr(r->ptr[0]) + chunk_off, chunk_bytes);
  const rsrc_t ro = make_rsrc(uni_ptr(r->ptr[3]) + chunk_off, chunk_bytes);
  // second / third input: laid out like x (K_FULL) or a [period, n] block reused every period rows;
  // layer norm: gamma and beta are always one row
  rsrc_t rs[2];
  uint32_t period[2] = {0, 0};
#pragma unroll
  for (int k = 1; k < RO::NIN; ++k) {
    if (!RO::SOFTMAX) {
      rs[k - 1] = make_rsrc(uni_ptr(r->ptr[k]), n * (P32 ? 4u : (uint32_t)E::ES));
    } else if (uni(r->okind[k]) == K_FULL) {
      rs[k - 1] = make_rsrc(uni_ptr(r->ptr[k]) + chunk_off, chunk_bytes);
    } else {
      period[k - 1] = uni(r->stride[k][0]);
      rs[k - 1] = make_rsrc(uni_ptr(r->ptr[k]), period[k - 1] * n * E::ES);
    }
  }
  // layer norm: this lane's pieces of gamma and beta are loaded once
  RowParam<POL, DT, P32> gq[KW], bq[KW];
  if (!RO::SOFTMAX) {
#pragma unroll
    for (int k = 0; k < KW; ++k) {
      const uint32_t vec = j + 64u * k;
      gq[k].load(rs[0], vec);                        // past the row: reads zeros (bounds-checked), never used
      bq[k].load(rs[1], vec);
    }
  }
  for (uint32_t base = row_begin + wave * rpw * UP; base < row_end; base += 4u * rpw * UP) {
    v4i q[UP][KW], mq[UP][KW];
    bool act[UP][KW];
#pragma unroll
    for (int u = 0; u < UP; ++u) {
      const uint32_t row = base + u * rpw + sub, lr = row - row_begin;
      uint32_t mr = lr;
      if (ROP == GPUOS_IMPL_MASKED_SOFTMAX_LAST && period[0]) mr = row % period[0];
#pragma unroll
      for (int k = 0; k < KW; ++k) {
        const uint32_t vec = j + 64u * k;
        act[u][k] = row < row_end && vec < vpr;
        // rows past the chunk and vectors past the row read zeros or a neighbour's data; masked below
        q[u][k] = M::ld16(rx, (lr * vpr + vec) * 16u);
        if (ROP == GPUOS_IMPL_MASKED_SOFTMAX_LAST) mq[u][k] = M::ld16(rs[0], (mr * vpr + vec) * 16u);
      }
    }
#pragma unroll
    for (int u = 0; u < UP; ++u) {
      const uint32_t row = base + u * rpw + sub, lr = row - row_begin;
      float t[KW][V];
      if (RO::SOFTMAX) {
        float m = -__builtin_inff();
#pragma unroll
        for (int k = 0; k < KW; ++k)
#pragma unroll
          for (int e = 0; e < (int)V; ++e) {
            float x = E::get(q[u][k], e);
            if (ROP == GPUOS_IMPL_MASKED_SOFTMAX_LAST) x = alpha * x + E::get(mq[u][k], e);
            t[k][e] = act[u][k] ? x : -__builtin_inff();
            m = __builtin_fmaxf(m, t[k][e]);
          }
        m = bfly_max(m, P);
        float s = 0.0f;
#pragma unroll
        for (int k = 0; k < KW; ++k)
#pragma unroll
          for (int e = 0; e < (int)V; ++e) { t[k][e] = __expf(t[k][e] - m); s += t[k][e]; }
        s = bfly_sum(s, P);
        const float inv = 1.0f / s;
#pragma unroll
        for (int k = 0; k < KW; ++k) {
          v4i oq;
#pragma unroll
          for (int e = 0; e < (int)V; ++e) E::put(oq, e, t[k][e] * inv);
          if (act[u][k]) M::st16(ro, (lr * vpr + j + 64u * k) * 16u, oq);
        }
      } else {
        float s = 0.0f;
#pragma unroll
        for (int k = 0; k < KW; ++k)
#pragma unroll
          for (int e = 0; e < (int)V; ++e) { t[k][e] = act[u][k] ? E::get(q[u][k], e) : 0.0f; s += t[k][e]; }
        const float mean = bfly_sum(s, P) / (float)n;
        float ss = 0.0f;
#pragma unroll
        for (int k = 0; k < KW; ++k)
#pragma unroll
          for (int e = 0; e < (int)V; ++e) { t[k][e] = act[u][k] ? t[k][e] - mean : 0.0f; ss += t[k][e] * t[k][e]; }
        const float var = bfly_sum(ss, P) / (float)n;
        const float rstd = 1.0f / __builtin_sqrtf(var + alpha);
#pragma unroll
        for (int k = 0; k < KW; ++k) {
          v4i oq;
#pragma unroll
          for (int e = 0; e < (int)V; ++e) E::put(oq, e, t[k][e] * rstd * gq[k].get(e) + bq[k].get(e));
          if (act[u][k]) M::st16(ro, (lr * vpr + j + 64u * k) * 16u, oq);
        }
      }
    }
  }
}

template <int POL, int ROP>
PATHFN void rowop_generic(const Record* r_v, uint32_t begin_v, uint32_t end_v) {
  const Record* r = lds_arg(r_v);
  const uint32_t row_begin = uni(begin_v), row_end = uni(end_v);
  using RO = RowOp<ROP>;
  const int nd = (int)uni(r->ndim);                   // outer dims
  const uint32_t n = uni(r->red_n);
  const float alpha = r->alpha;
  const char* p[3];
  uint32_t dt[3], sl[3];
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    const int kk = k < RO::NIN ? k : 0;
    p[k] = uni_ptr(r->ptr[kk]); dt[k] = uni(r->dtype[kk]); sl[k] = uni(r->stride[kk][5]);
  }
  char* po = (char*)uni_ptr(r->ptr[3]);
  const uint32_t odt = uni(r->dtype[3]), slo = uni(r->stride[3][5]);
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  for (uint32_t row = row_begin + wave; row < row_end; row += 4) {
    uint32_t rem = row, off[3] = {0, 0, 0}, ooff = 0;
#pragma unroll
    for (int d = GPUOS_MAX_DIMS - 2; d >= 0; --d) {
      if (d < nd) {
        const uint32_t sz = uni(r->size[d]);
        const uint32_t qd = rem / sz, idx = rem - qd * sz;
        rem = qd;
#pragma unroll
        for (int k = 0; k < RO::NIN; ++k) off[k] += idx * uni(r->stride[k][d]);
        ooff += idx * uni(r->stride[3][d]);
      }
    }
    if (RO::SOFTMAX) {
      auto arg = [&](uint32_t jx) {
        float x = load_rt<POL>(p[0], off[0] + jx * sl[0], dt[0]);
        if (ROP == GPUOS_IMPL_MASKED_SOFTMAX_LAST) x = alpha * x + load_rt<POL>(p[1], off[1] + jx * sl[1], dt[1]);
        return x;
      };
      float m = -__builtin_inff();
      for (uint32_t jx = lane; jx < n; jx += 64) m = __builtin_fmaxf(m, arg(jx));
      m = bfly_max(m, 64);
      float s = 0.0f;
      for (uint32_t jx = lane; jx < n; jx += 64) s += __expf(arg(jx) - m);
      s = bfly_sum(s, 64);
      const float inv = 1.0f / s;
      for (uint32_t jx = lane; jx < n; jx += 64) store_rt<POL>(po, ooff + jx * slo, odt, __expf(arg(jx) - m) * inv);
    } else {
      float s = 0.0f;
      for (uint32_t jx = lane; jx < n; jx += 64) s += load_rt<POL>(p[0], off[0] + jx * sl[0], dt[0]);
      const float mean = bfly_sum(s, 64) / (float)n;
      float ss = 0.0f;
      for (uint32_t jx = lane; jx < n; jx += 64) {
        const float d = load_rt<POL>(p[0], off[0] + jx * sl[0], dt[0]) - mean;
        ss += d * d;
      }
      const float var = bfly_sum(ss, 64) / (float)n;
      const float rstd = 1.0f / __builtin_sqrtf(var + alpha);
      for (uint32_t jx = lane; jx < n; jx += 64) {
        const float d = load_rt<POL>(p[0], off[0] + jx * sl[0], dt[0]) - mean;
        store_rt<POL>(po, ooff + jx * slo, odt,
                      d * rstd * load_rt<POL>(p[1], off[1] + jx * sl[1], dt[1]) + load_rt<POL>(p[2], off[2] + jx * sl[2], dt[2]));
      }
    }
  }
}

// Rows longer than one wavefront's registers: the whole workgroup owns a row.  KW = 1..4: the row
// (up to 1024 vectors) lives in registers, 256 lanes x KW vectors, read once and written once.
// KW = 0: any length, three streaming passes of 16-byte vector loads over the row (the second and
// third pass re-read what the first brought into the caches).  Cross-wavefront reductions go
// through four rotating LDS slots: one barrier per reduction.
template <int POL, int ROP, int DT, int KW, bool P32 = false>
DEV void rowop_wg(const Record* r, uint32_t row_begin, uint32_t row_end, float* s_red) {
  using E = Elem<DT>;
  using M = Mem<POL>;
  using RO = RowOp<ROP>;
  constexpr uint32_t V = E::V;
  constexpr int KR = KW > 0 ? KW : 1;
  const uint32_t n = uni(r->red_n), vpr = n / V;
  const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  const float alpha = r->alpha;
  const uint32_t nrows = row_end - row_begin;
  const uint32_t chunk_bytes = nrows * n * E::ES;
  const uint64_t chunk_off = (uint64_t)row_begin * n * E::ES;
  const rsrc_t rx = make_rsrc(uni_ptr(r->ptr[0]) + chunk_off, chunk_bytes);
  const rsrc_t ro = make_rsrc(uni_ptr(r->ptr[3]) + chunk_off, chunk_bytes);
  rsrc_t rs[2];
  uint32_t period[2] = {0, 0};
#pragma unroll
  for (int k = 1; k < RO::NIN; ++k) {
    if (!RO::SOFTMAX) {
      rs[k - 1] = make_rsrc(uni_ptr(r->ptr[k]), n * (P32 ? 4u : (uint32_t)E::ES));      // gamma, beta: one row
    } else if (uni(r->okind[k]) == K_FULL) {
      rs[k - 1] = make_rsrc(uni_ptr(r->ptr[k]) + chunk_off, chunk_bytes);
    } else {
      period[k - 1] = uni(r->stride[k][0]);
      rs[k - 1] = make_rsrc(uni_ptr(r->ptr[k]), period[k - 1] * n * E::ES);
    }
  }
  uint32_t turn = 0;                                   // which of the four LDS slots the next reduction uses
  auto wg_sum = [&](float v) {
    v = bfly_sum(v, 64);
    float* slot = s_red + (turn & 3u) * 4u;
    ++turn;
    if (lane == 0) slot[wave] = v;
    __syncthreads();
    return (slot[0] + slot[1]) + (slot[2] + slot[3]);
  };
  auto wg_max = [&](float v) {
    v = bfly_max(v, 64);
    float* slot = s_red + (turn & 3u) * 4u;
    ++turn;
    if (lane == 0) slot[wave] = v;
    __syncthreads();
    return __builtin_fmaxf(__builtin_fmaxf(slot[0], slot[1]), __builtin_fmaxf(slot[2], slot[3]));
  };
  // the argument of element e of vector `vec` of local row lr (softmax family) / the element itself
  auto arg = [&](const v4i& q, const v4i& mq, int e) {
    float x = E::get(q, e);
    if (ROP == GPUOS_IMPL_MASKED_SOFTMAX_LAST) x = alpha * x + E::get(mq, e);
    return x;
  };
  RowParam<POL, DT, P32> gq[KR], bq[KR];               // layer norm, KW > 0: this lane's gamma / beta pieces
  if (!RO::SOFTMAX && KW > 0) {
#pragma unroll
    for (int k = 0; k < KR; ++k) {
      gq[k].load(rs[0], tid + kThreads * k);
      bq[k].load(rs[1], tid + kThreads * k);
    }
  }
  for (uint32_t row = row_begin; row < row_end; ++row) {
    const uint32_t lr = row - row_begin;
    uint32_t mr = lr;
    if (ROP == GPUOS_IMPL_MASKED_SOFTMAX_LAST && period[0]) mr = row % period[0];
    if (KW > 0) {
      v4i q[KR], mq[KR];
      bool act[KR];
#pragma unroll
      for (int k = 0; k < KR; ++k) {
        const uint32_t vec = tid + kThreads * k;
        act[k] = vec < vpr;
        q[k] = M::ld16(rx, act[k] ? (lr * vpr + vec) * 16u : kNoLoad);
        if (ROP == GPUOS_IMPL_MASKED_SOFTMAX_LAST) mq[k] = M::ld16(rs[0], act[k] ? (mr * vpr + vec) * 16u : kNoLoad);
      }
      float t[KR][V];
      if (RO::SOFTMAX) {
        float m = -__builtin_inff();
#pragma unroll
        for (int k = 0; k < KR; ++k)
#pragma unroll
          for (int e = 0; e < (int)V; ++e) { t[k][e] = act[k] ? arg(q[k], mq[k], e) : -__builtin_inff(); m = __builtin_fmaxf(m, t[k][e]); }
        m = wg_max(m);
        float sum = 0.0f;
#pragma unroll
        for (int k = 0; k < KR; ++k)
#pragma unroll
          for (int e = 0; e < (int)V; ++e) { t[k][e] = __expf(t[k][e] - m); sum += t[k][e]; }
        const float inv = 1.0f / wg_sum(sum);
#pragma unroll
        for (int k = 0; k < KR; ++k) {
          v4i oq;
#pragma unroll
          for (int e = 0; e < (int)V; ++e) E::put(oq, e, t[k][e] * inv);
          if (act[k]) M::st16(ro, (lr * vpr + tid + kThreads * k) * 16u, oq);
        }
      } else {
        float sum = 0.0f;
#pragma unroll
        for (int k = 0; k < KR; ++k)
#pragma unroll
          for (int e = 0; e < (int)V; ++e) { t[k][e] = act[k] ? E::get(q[k], e) : 0.0f; sum += t[k][e]; }
        const float mean = wg_sum(sum) / (float)n;
        float ss = 0.0f;
#pragma unroll
        for (int k = 0; k < KR; ++k)
#pragma unroll
          for (int e = 0; e < (int)V; ++e) { t[k][e] = act[k] ? t[k][e] - mean : 0.0f; ss += t[k][e] * t[k][e]; }
        const float rstd = 1.0f / __builtin_sqrtf(wg_sum(ss) / (float)n + alpha);
#pragma unroll
        for (int k = 0; k < KR; ++k) {
          v4i oq;
#pragma unroll
          for (int e = 0; e < (int)V; ++e) E::put(oq, e, t[k][e] * rstd * gq[k].get(e) + bq[k].get(e));
          if (act[k]) M::st16(ro, (lr * vpr + tid + kThreads * k) * 16u, oq);
        }
      }
    } else if (RO::SOFTMAX) {
      const v4i zero = {0, 0, 0, 0};
      float m = -__builtin_inff();
      for (uint32_t vec = tid; vec < vpr; vec += kThreads) {
        const v4i q = M::ld16(rx, (lr * vpr + vec) * 16u);
        const v4i mq = ROP == GPUOS_IMPL_MASKED_SOFTMAX_LAST ? M::ld16(rs[0], (mr * vpr + vec) * 16u) : zero;
#pragma unroll
        for (int e = 0; e < (int)V; ++e) m = __builtin_fmaxf(m, arg(q, mq, e));
      }
      m = wg_max(m);
      float sum = 0.0f;
      for (uint32_t vec = tid; vec < vpr; vec += kThreads) {
        const v4i q = M::ld16(rx, (lr * vpr + vec) * 16u);
        const v4i mq = ROP == GPUOS_IMPL_MASKED_SOFTMAX_LAST ? M::ld16(rs[0], (mr * vpr + vec) * 16u) : zero;
#pragma unroll
        for (int e = 0; e < (int)V; ++e) sum += __expf(arg(q, mq, e) - m);
      }
      const float inv = 1.0f / wg_sum(sum);
      for (uint32_t vec = tid; vec < vpr; vec += kThreads) {
        const v4i q = M::ld16(rx, (lr * vpr + vec) * 16u);
        const v4i mq = ROP == GPUOS_IMPL_MASKED_SOFTMAX_LAST ? M::ld16(rs[0], (mr * vpr + vec) * 16u) : zero;
        v4i oq;
#pragma unroll
        for (int e = 0; e < (int)V; ++e) E::put(oq, e, __expf(arg(q, mq, e) - m) * inv);
        M::st16(ro, (lr * vpr + vec) * 16u, oq);
      }
    } else {
      float sum = 0.0f;
      for (uint32_t vec = tid; vec < vpr; vec += kThreads) {
        const v4i q = M::ld16(rx, (lr * vpr + vec) * 16u);
#pragma unroll
        for (int e = 0; e < (int)V; ++e) sum += E::get(q, e);
      }
      const float mean = wg_sum(sum) / (float)n;
      float ss = 0.0f;
      for (uint32_t vec = tid; vec < vpr; vec += kThreads) {
        const v4i q = M::ld16(rx, (lr * vpr + vec) * 16u);
#pragma unroll
        for (int e = 0; e < (int)V; ++e) { const float d = E::get(q, e) - mean; ss += d * d; }
      }
      const float rstd = 1.0f / __builtin_sqrtf(wg_sum(ss) / (float)n + alpha);
      for (uint32_t vec = tid; vec < vpr; vec += kThreads) {
        const v4i q = M::ld16(rx, (lr * vpr + vec) * 16u);
        RowParam<POL, DT, P32> g, b;
        g.load(rs[0], vec);
        b.load(rs[1], vec);
        v4i oq;
#pragma unroll
        for (int e = 0; e < (int)V; ++e) E::put(oq, e, (E::get(q, e) - mean) * rstd * g.get(e) + b.get(e));
        M::st16(ro, (lr * vpr + vec) * 16u, oq);
      }
    }
  }
  __syncthreads();                                     // the LDS slots belong to the next chunk after this
}

template <int POL, int ROP, int DT>
PATHFN void rowop_fused_dt(const Record* r_v, uint32_t begin_v, uint32_t end_v) {
  const Record* r = lds_arg(r_v);
  const uint32_t begin = uni(begin_v), end = uni(end_v);
  const uint32_t vpr = uni(r->red_n) / Elem<DT>::V;
  if (ROP == GPUOS_IMPL_LAYERNORM_LAST && DT != GPUOS_F32 && uni(r->dtype[1]) == GPUOS_F32) {   // fp32 gamma / beta under 16-bit x
    constexpr bool P = ROP == GPUOS_IMPL_LAYERNORM_LAST && DT != GPUOS_F32;
    if (vpr <= 64u) rowop_fused<POL, ROP, DT, 1, 4, P>(r, begin, end);
    else if (vpr <= 128u) rowop_fused<POL, ROP, DT, 2, 2, P>(r, begin, end);
    else rowop_fused<POL, ROP, DT, 4, 1, P>(r, begin, end);
    return;
  }
  if (vpr <= 64u) rowop_fused<POL, ROP, DT, 1, 4>(r, begin, end);
  else if (vpr <= 128u) rowop_fused<POL, ROP, DT, 2, 2>(r, begin, end);
  else rowop_fused<POL, ROP, DT, 4, 1>(r, begin, end);
}

template <int POL, int ROP, int DT>
PATHFN void rowop_wg_dt(const Record* r_v, uint32_t begin_v, uint32_t end_v, float* s_v) {
  const Record* r = lds_arg(r_v);
  float* s_red = lds_arg(s_v);
  const uint32_t begin = uni(begin_v), end = uni(end_v);
  const uint32_t vpr = uni(r->red_n) / Elem<DT>::V;
  if (ROP == GPUOS_IMPL_LAYERNORM_LAST && DT != GPUOS_F32 && uni(r->dtype[1]) == GPUOS_F32) {
    constexpr bool P = ROP == GPUOS_IMPL_LAYERNORM_LAST && DT != GPUOS_F32;
    if (vpr <= 512u) rowop_wg<POL, ROP, DT, 2, P>(r, begin, end, s_red);
    else if (vpr <= 1024u) rowop_wg<POL, ROP, DT, 4, P>(r, begin, end, s_red);
    else rowop_wg<POL, ROP, DT, 0, P>(r, begin, end, s_red);
    return;
  }
  if (vpr <= 512u) rowop_wg<POL, ROP, DT, 2>(r, begin, end, s_red);
  else if (vpr <= 1024u) rowop_wg<POL, ROP, DT, 4>(r, begin, end, s_red);
  else rowop_wg<POL, ROP, DT, 0>(r, begin, end, s_red);
}

template <int POL, int ROP>
DEV void run_rowop(const Record* r, uint32_t chunk, float* s_red) {
  const uint32_t per = uni(r->chunk), rows = uni(r->numel);
  const uint32_t begin = chunk * per;
  const uint32_t end = (rows - begin < per) ? rows : begin + per;
  if (uni(r->path) == PATH_ROW_FUSED) {
    const uint32_t dt = uni(r->dtype[3]);
    const bool wide = uni(r->red_n) * (dt == GPUOS_F32 ? 4u : 2u) > 256u * 16u;     // more than 256 vectors per row
    if (!wide) {
      if (dt == GPUOS_F32) rowop_fused_dt<POL, ROP, GPUOS_F32>(r, begin, end);
      else if (dt == GPUOS_F16) rowop_fused_dt<POL, ROP, GPUOS_F16>(r, begin, end);
      else rowop_fused_dt<POL, ROP, GPUOS_BF16>(r, begin, end);
    } else {
      if (dt == GPUOS_F32) rowop_wg_dt<POL, ROP, GPUOS_F32>(r, begin, end, s_red);
      else if (dt == GPUOS_F16) rowop_wg_dt<POL, ROP, GPUOS_F16>(r, begin, end, s_red);
      else rowop_wg_dt<POL, ROP, GPUOS_BF16>(r, begin, end, s_red);
    }
  } else {
    rowop_generic<POL, ROP>(r, begin, end);
  }
}

// ---------------------------------------------------------------------------
// chunk executor: operator dispatch by implementation id (the role of the
// paper's function-pointer table call, Section 4.1; here a switch over
// precompiled implementations selected by the table entry).
// ---------------------------------------------------------------------------
template <int POL, int IMPL>
DEV void run_elementwise(const Record* r, uint32_t chunk, float* s_scratch) {
  const uint32_t per = uni(r->chunk), numel = uni(r->numel);
  const uint32_t begin = chunk * per;
  const uint32_t end = (numel - begin < per) ? numel : begin + per;
  const uint32_t path = uni(r->path), dt = uni(r->dtype[3]);
  constexpr bool int_ok = IMPL == GPUOS_IMPL_ADD || IMPL == GPUOS_IMPL_SUB || IMPL == GPUOS_IMPL_MUL || IMPL == GPUOS_IMPL_COPY;
  if (r->rflags & RF_INT) {
    if (int_ok) {
      if (path == PATH_CONTIG) ew_contig_int<POL, IMPL>(r, begin, end);
      else ew_generic<POL, int_ok ? IMPL : GPUOS_IMPL_COPY, true>(r, begin, end);
    }
    return;
  }
  if (path == PATH_CONTIG) {
    if (dt == GPUOS_F32) ew_contig<POL, IMPL, GPUOS_F32>(r, begin, end);
    else if (dt == GPUOS_F16) ew_contig<POL, IMPL, GPUOS_F16>(r, begin, end);
    else ew_contig<POL, IMPL, GPUOS_BF16>(r, begin, end);
  } else if (path == PATH_ROW2D && Op<IMPL>::N >= 2) {
    constexpr int I2 = Op<IMPL>::N >= 2 ? IMPL : GPUOS_IMPL_ADD;
    const uint32_t k0 = uni(r->okind[0]), k1 = uni(r->okind[1]);
    const int spec = (Op<I2>::N == 2 && k0 == K_FULL) ? (k1 == K_ROWSCALAR ? 1 : (k1 == K_ROWVEC ? 2 : 0)) : 0;
    if (dt == GPUOS_F32) {
      if (spec == 1) ew_row2d<POL, I2, GPUOS_F32, K_ROWSCALAR>(r, begin, end, s_scratch);
      else if (spec == 2) ew_row2d<POL, I2, GPUOS_F32, K_ROWVEC>(r, begin, end, s_scratch);
      else ew_row2d<POL, I2, GPUOS_F32, -1>(r, begin, end, s_scratch);
    } else if (dt == GPUOS_F16) {
      if (spec == 1) ew_row2d<POL, I2, GPUOS_F16, K_ROWSCALAR>(r, begin, end, s_scratch);
      else if (spec == 2) ew_row2d<POL, I2, GPUOS_F16, K_ROWVEC>(r, begin, end, s_scratch);
      else ew_row2d<POL, I2, GPUOS_F16, -1>(r, begin, end, s_scratch);
    } else {
      if (spec == 1) ew_row2d<POL, I2, GPUOS_BF16, K_ROWSCALAR>(r, begin, end, s_scratch);
      else if (spec == 2) ew_row2d<POL, I2, GPUOS_BF16, K_ROWVEC>(r, begin, end, s_scratch);
      else ew_row2d<POL, I2, GPUOS_BF16, -1>(r, begin, end, s_scratch);
    }
  } else if (path == PATH_TILE2D) {
    ew_tile2d<POL, IMPL>(r, begin, end, s_scratch);      // begin / end count tiles here
  } else if (path == PATH_STAGED) {
    ew_staged<POL, IMPL>(r, begin, end, s_scratch);
  } else {
    ew_generic<POL, IMPL, false>(r, begin, end);
  }
}

template <int POL, int RIMPL>
DEV void run_reduction(const Record* r, uint32_t chunk, float* s_red) {
  const uint32_t per = uni(r->chunk), rows = uni(r->numel);
  const uint32_t begin = chunk * per;
  const uint32_t end = (rows - begin < per) ? rows : begin + per;
  const uint32_t path = uni(r->path), dt = uni(r->dtype[0]);
  if (r->rflags & RF_INT) { red_generic<POL, RIMPL, true>(r, begin, end); return; }
  if (path == PATH_RED_CONTIG) {
    if (dt == GPUOS_F32) red_contig<POL, RIMPL, GPUOS_F32>(r, begin, end, s_red);
    else if (dt == GPUOS_F16) red_contig<POL, RIMPL, GPUOS_F16>(r, begin, end, s_red);
    else red_contig<POL, RIMPL, GPUOS_BF16>(r, begin, end, s_red);
  } else {
    red_generic<POL, RIMPL, false>(r, begin, end);
  }
}

// A task whose operator is a program: fetch the program into LDS (17 lanes x 16 bytes), then run
// the ordinary elementwise paths with the interpreter as their functor.
template <int POL>
DEV int32_t exec_program(const Record* r, uint32_t impl, uint32_t chunk, float* s_red, const ProgramImage* progs) {
  const uint32_t k = impl - GPUOS_IMPL_PROGRAM_BASE;
  if (progs == nullptr || k >= GPUOS_MAX_PROGRAMS) return GPUOS_E_BADOP;
  const rsrc_t rp = make_rsrc(progs + k, (uint32_t)sizeof(ProgramImage));
  if (threadIdx.x < sizeof(ProgramImage) / 16) ((v4i*)&g_prog)[threadIdx.x] = Mem<POL_COHERENT>::ld16(rp, threadIdx.x * 16u);
  __syncthreads();
  int32_t status = GPUOS_OK;
  const uint32_t n_in = uni(g_prog.n_inputs), n_instr = uni(g_prog.n_instr);
  if (uni(g_prog.ready) != kProgramReady || n_instr < 1 || n_instr > GPUOS_PROGRAM_MAX_INSTR || n_in != uni(r->n_inputs))
    status = GPUOS_E_INVAL;                            // never defined (or not what the task was packed for)
  else if (n_in == 1) run_elementwise<POL, kImplProg1>(r, chunk, s_red);
  else if (n_in == 2) run_elementwise<POL, kImplProg2>(r, chunk, s_red);
  else run_elementwise<POL, kImplProg3>(r, chunk, s_red);
  __syncthreads();                                     // the next chunk may bring another program
  return status;
}

// returns the task status contribution of this chunk (0 or an error)
template <int POL>
DEV int32_t exec_chunk(const Record* r, uint32_t impl, uint32_t chunk, float* s_red, const ProgramImage* progs) {
  if (uni(r->path) == PATH_NOP) return impl == GPUOS_IMPL_FAIL ? GPUOS_E_BADOP : GPUOS_OK;
  if (impl >= GPUOS_IMPL_PROGRAM_BASE) return exec_program<POL>(r, impl, chunk, s_red, progs);
  switch (impl) {
    case GPUOS_IMPL_ADD: run_elementwise<POL, GPUOS_IMPL_ADD>(r, chunk, s_red); break;
    case GPUOS_IMPL_SUB: run_elementwise<POL, GPUOS_IMPL_SUB>(r, chunk, s_red); break;
    case GPUOS_IMPL_MUL: run_elementwise<POL, GPUOS_IMPL_MUL>(r, chunk, s_red); break;
    case GPUOS_IMPL_DIV: run_elementwise<POL, GPUOS_IMPL_DIV>(r, chunk, s_red); break;
    case GPUOS_IMPL_RELU: run_elementwise<POL, GPUOS_IMPL_RELU>(r, chunk, s_red); break;
    case GPUOS_IMPL_EXP: run_elementwise<POL, GPUOS_IMPL_EXP>(r, chunk, s_red); break;
    case GPUOS_IMPL_GELU_ERF: run_elementwise<POL, GPUOS_IMPL_GELU_ERF>(r, chunk, s_red); break;
    case GPUOS_IMPL_GELU_TANH: run_elementwise<POL, GPUOS_IMPL_GELU_TANH>(r, chunk, s_red); break;
    case GPUOS_IMPL_SCALE: run_elementwise<POL, GPUOS_IMPL_SCALE>(r, chunk, s_red); break;
    case GPUOS_IMPL_FMA: run_elementwise<POL, GPUOS_IMPL_FMA>(r, chunk, s_red); break;
    case GPUOS_IMPL_SUB_EXP: run_elementwise<POL, GPUOS_IMPL_SUB_EXP>(r, chunk, s_red); break;
    case GPUOS_IMPL_COPY: run_elementwise<POL, GPUOS_IMPL_COPY>(r, chunk, s_red); break;
    case GPUOS_IMPL_SUM_LAST: run_reduction<POL, GPUOS_IMPL_SUM_LAST>(r, chunk, s_red); break;
    case GPUOS_IMPL_MAX_LAST: run_reduction<POL, GPUOS_IMPL_MAX_LAST>(r, chunk, s_red); break;
    case GPUOS_IMPL_MIN_LAST: run_reduction<POL, GPUOS_IMPL_MIN_LAST>(r, chunk, s_red); break;
    case GPUOS_IMPL_SOFTMAX_LAST: run_rowop<POL, GPUOS_IMPL_SOFTMAX_LAST>(r, chunk, s_red); break;
    case GPUOS_IMPL_MASKED_SOFTMAX_LAST: run_rowop<POL, GPUOS_IMPL_MASKED_SOFTMAX_LAST>(r, chunk, s_red); break;
    case GPUOS_IMPL_LAYERNORM_LAST: run_rowop<POL, GPUOS_IMPL_LAYERNORM_LAST>(r, chunk, s_red); break;
    case GPUOS_IMPL_FAIL: return GPUOS_E_BADOP;       // kill-switch stub: fail fast, write nothing
    default: return GPUOS_E_BADOP;
  }
  return GPUOS_OK;
}


// Reading the clock is a memory-like operation: a dozen reads per task are measurable, so the phase
// timers are an option and the clock is read only where something needs the value.
DEV uint64_t clock_if(bool on) { return on ? wall_clock64() : 0ull; }

// The 16 lanes that hold a record's 16-byte pieces: the weighted check sum of the whole record
// (see record_check_weight), in every one of them.

DEV uint32_t record_piece_sum(const v4i& q, uint32_t part) {
  uint32_t x = 0;
#pragma unroll
  for (uint32_t j = 0; j < 4; ++j) x += (uint32_t)q[j] * record_check_weight(4u * part + j);
  // sum over the 16 lanes of the row with DPP rotations (row_ror 8, 4, 2, 1): every lane ends with
  // the whole sum, and unlike a shuffle nothing goes through the LDS crossbar
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x128, 0xf, 0xf, false);
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x124, 0xf, 0xf, false);
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x122, 0xf, 0xf, false);
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x121, 0xf, 0xf, false);
  return x;
}

struct BuiltinExec {                // what the library's own workers execute a chunk with
  static DEV int32_t run(const Record* r, uint32_t impl, uint32_t chunk, float* s_red, const ProgramImage* progs) {
    return exec_chunk<POL_COHERENT>(r, impl, chunk, s_red, progs);
  }
};

// ---------------------------------------------------------------------------
// worker (every workgroup but 0)
// ---------------------------------------------------------------------------
constexpr uint32_t kMirrorRetries = 1u << 22;       // fetches of a mirror record that does not (yet) verify: seconds
constexpr uint64_t kStopGraceTicks = 10000000ull;   // 100 ms (100 MHz clock): how long a worker still waits for a dependency once the stop flag is up

// A workgroup holds up to kStash descriptors: work units it has claimed that wait for a dependency,
// and the one it runs.  A workgroup whose unit must wait does not sit on it: it claims the next
// unit and runs whatever it holds that is ready (oldest first).  A chain of dependent small tasks
// then occupies one descriptor slot per link in flight instead of one whole workgroup, so eight
// times as many chains are in flight (Section 6.1's sequences issued one after the other: 1.7 M ->
// see the benchmark).  Progress: units are claimed in publication order and what a waiting unit names
// was published before it, so the unfinished unit with the lowest number is always held by some
// workgroup with nothing left to wait for, and every workgroup looks at everything it holds on every
// poll.
constexpr uint32_t kStash = 8;
constexpr uint32_t kStashFull = (1u << kStash) - 1u;
enum : uint32_t { kActRun = 0, kActFetch = 1, kActExit = 2 };

struct WorkShared {
  Record rec[kStash];              // descriptors held
  uint64_t unit[kStash];           // their work-unit entries
  uint64_t entry[kStash];          // the operator-table slot each one claimed
  uint64_t since[kStash];          // when each began to wait (device clock)
  uint32_t action, slot;           // the first wavefront's decision: run the unit in descriptor slot `slot`, fetch
                                   // the newly claimed unit's descriptor into it, or leave
  int32_t dep_status;              // 0, or the status a task whose dependency wait ran out completes with
  uint32_t rec_sum;                // weighted check sum of the record as fetched
  alignas(16) float red[kScratchFloats];   // (16-byte LDS vectors are written into it)
};

DEV uint64_t uni64(uint64_t v) {
  return ((uint64_t)__builtin_amdgcn_readfirstlane((uint32_t)(v >> 32)) << 32) | __builtin_amdgcn_readfirstlane((uint32_t)v);
}
DEV uint64_t lane64(uint64_t v, uint32_t lane) {     // `lane` the same in every lane
  return ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), (int)lane) << 32) |
         (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, (int)lane);
}

// First wavefront: fetch the descriptor that work unit `unit` names (16 lanes x 16 bytes) and the
// operator-table slot it claimed into descriptor slot f, with the record's weighted check sum.
DEV void fetch_descriptor(const WorkerArgs& a, WorkShared* s, rsrc_t rd, uint64_t unit, uint32_t f) {
  const uint32_t tid = threadIdx.x;
  const uint32_t slot = (uint32_t)((unit >> 20) & 0xffffu);
  const uint32_t op = (uint32_t)((unit >> 36) & 0xffu), sel = (uint32_t)((unit >> 44) & 1u);
  const bool op_valid = ((unit >> 45) & 1u) != 0;
  v4i q = {0, 0, 0, 0};
  uint64_t ent = 0;
  if (tid < 16) q = Mem<POL_COHERENT>::ld16(rd, slot * (uint32_t)sizeof(Record) + tid * 16u);
  if (tid == 16 && op_valid) ent = __hip_atomic_load(&a.dtable[op].slot[sel], __ATOMIC_RELAXED, SC_SYSTEM);
  const uint32_t x = record_piece_sum(q, tid & 15u);
  if (tid < 16) ((v4i*)&s->rec[f])[tid] = q;
  if (tid == 16) s->entry[f] = ent;
  if (tid == 0) s->rec_sum = x;
}

// RING 0: the library's own workers, on the main unit ring, executing through EXEC = the built-in
// chunk executor.  RING 1: the workers of a kernel compiled at run time, on the second unit ring
// (the dispatcher routes the tasks of natively compiled operator programs there), executing through
// the EXEC that kernel brings; `gen` is the generation of that kernel: its workers leave when the
// host asks for a later one.
template <int RING, class EXEC>
DEV void run_worker(const WorkerArgs& a, WorkShared* s, uint32_t gen = 0) {
  const uint32_t tid = threadIdx.x;
  uint64_t* const claim_ctr = RING == 0 ? &a.d->claim : &a.d->claim_j;
  const uint64_t* const unit_ring = RING == 0 ? a.units : a.units_j;
  const rsrc_t rd = make_rsrc(a.dring, (a.cap_mask + 1u) * (uint32_t)sizeof(Record));
  uint64_t w_units = 0, w_wait = 0, w_fetch = 0, w_dep = 0, w_exec = 0, w_done = 0;
  const bool timing = a.timing != 0, tracing = a.trace != nullptr;
  const uint64_t w_start = clock_if(timing);
  // State of the first wavefront (the same in all its lanes; the other wavefronts never look at it).
  uint32_t waiting = 0;            // bit k: descriptor slot k holds a unit that waits for a dependency
  bool have_claim = false;         // a unit number is claimed and its entry has not arrived yet
  bool draining = false;           // the stop flag was seen: claim nothing more, finish what is held, leave
  uint64_t g = 0;                  // the claimed unit number
  uint32_t polls = 0, yield_every = 0;
  while (true) {
    const uint64_t c0 = clock_if(timing);
    const bool held_any = waiting != 0;
    // ---- decide what to do next (first wavefront): one round of loads per poll ----
    // Lane 32 polls the claimed entry itself (its stamp is the ready flag: every waiting workgroup
    // polls a different address); lane k < kStash looks at the done words that descriptor slot k waits for.
    if (tid < 64) {
      uint32_t action = kActExit, f = 0;
      int32_t dep_status = 0;
      uint64_t u_new = 0;
      if (!have_claim && !draining && waiting != kStashFull) {
        uint64_t gg = 0;
        if (tid == 0) gg = __hip_atomic_fetch_add(claim_ctr, 1ull, __ATOMIC_RELAXED, SC_AGENT);
        g = uni64(gg);
        have_claim = true;
        polls = 0;
      }
      const uint64_t* up = &unit_ring[g & a.unit_mask];
      const uint64_t want = unit_stamp(g, a.unit_shift);
      // What is awaited was published before the unit that waits (the dispatcher sees to that), so the
      // wait ends when resident workgroups finish work they hold.  It is bounded all the same (the
      // context's wait limit; a short grace once the stop flag is up): a task that runs into the
      // bound completes with GPUOS_E_TIMEOUT without executing, and the kernel always leaves.
      const bool mine = tid < kStash && ((waiting >> tid) & 1u);
      uint64_t need[3] = {0ull, 0ull, 0ull};
      const uint64_t* done_word[3] = {nullptr, nullptr, nullptr};
      if (mine) {
        const Record* r = &s->rec[tid];
        const uint64_t ticket = r->ticket;
#pragma unroll
        for (int k = 0; k < 3; ++k) {
          const uint32_t back = r->dep[k];
          if (back != 0 && back <= ticket) {
            need[k] = ticket - back + 1;
            done_word[k] = &a.st[(ticket - back) & a.cap_mask].done_seq;
          }
        }
      }
      // One round of loads per poll.  (Keeping a second round in flight, to sample twice per memory
      // round trip, was measured: with 767 workgroups polling, the doubled traffic cost a lone task
      // more than the earlier sample gained, 7.7 against 6.5 us.)
      struct Poll { uint64_t u, seen[3]; };
      // While something is held, every lane issues all four loads, the lanes with nothing to look at from
      // the unit-ring entry that lane 32 polls anyway (one request for the whole wavefront): loads under
      // conditions that differ between lanes are waited for one after the other (a poll would take up
      // to four memory round trips instead of one).
      const uint64_t* const anyword = up;
      auto request = [&]() {
        Poll p;
        if (waiting == 0) {
          p.u = 0;
          if (tid == 32 && have_claim) p.u = __hip_atomic_load(up, __ATOMIC_RELAXED, SC_SYSTEM);
          p.seen[0] = p.seen[1] = p.seen[2] = ~0ull;
        } else {
          p.u = __hip_atomic_load(up, __ATOMIC_RELAXED, SC_SYSTEM);
#pragma unroll
          for (int k = 0; k < 3; ++k) p.seen[k] = __hip_atomic_load(done_word[k] ? done_word[k] : anyword, __ATOMIC_RELAXED, SC_SYSTEM);
        }
        return p;
      };
      while (true) {
        const Poll cur = request();
        bool ready = mine && cur.seen[0] >= need[0] && cur.seen[1] >= need[1] && cur.seen[2] >= need[2];
        int32_t gave_up = 0;
        if (mine && !ready && (polls & 31u) == 31u) {
          uint64_t limit = a.dep_wait_ticks;
          if (limit > kStopGraceTicks && __hip_atomic_load(&a.d->stop_dev, __ATOMIC_RELAXED, SC_SYSTEM)) limit = kStopGraceTicks;
          if (wall_clock64() - s->since[tid] > limit) { gave_up = GPUOS_E_TIMEOUT; ready = true; }
        }
        order_loads();
        const uint64_t m_ready = __ballot(ready);
        u_new = lane64(cur.u, 32u);
        if (m_ready != 0) {                                   // the first descriptor slot whose unit can run (any ready
          f = (uint32_t)__builtin_ctzll(m_ready);             // one makes progress)
          dep_status = __builtin_amdgcn_readlane(gave_up, (int)f);
          waiting &= ~(1u << f);
          action = kActRun;
          break;
        }
        if (have_claim && (u_new >> 46) == want) {
          f = (uint32_t)__builtin_ctz(~waiting);              // a free descriptor slot (claims are made only while one exists)
          have_claim = false;
          action = kActFetch;
          fetch_descriptor(a, s, rd, u_new, f);  // requested at once: the other wavefronts need not hear of the unit first
          break;
        }
        ++polls;
        if ((polls & 31u) == 0) {
          // (a run-time kernel also leaves when a later generation is wanted: the host asks for that
          // only once nothing is routed to this ring any more and everything routed has completed)
          const bool stop = __hip_atomic_load(&a.d->stop_dev, __ATOMIC_RELAXED, SC_SYSTEM) != 0 ||
                            (RING == 1 && __hip_atomic_load(&a.d->jit_gen, __ATOMIC_RELAXED, SC_SYSTEM) > gen);
          if (stop && !draining) {
            order_loads();                                    // every unit was stored before the stop flag
            if (have_claim) {
              u_new = uni64(__hip_atomic_load(up, __ATOMIC_RELAXED, SC_SYSTEM));
              order_loads();
              if ((u_new >> 46) == want) {
                f = (uint32_t)__builtin_ctz(~waiting);
                have_claim = false;
                action = kActFetch;
                fetch_descriptor(a, s, rd, u_new, f);
                break;
              }
              // The number claimed will never be served.  The second ring stays in use across
              // generations of run-time kernels while the dispatcher runs on: give the number back
              // (nothing is being published to that ring at this time, so the count ends exact).
              if (RING == 1 && tid == 0) __hip_atomic_fetch_add(claim_ctr, ~0ull, __ATOMIC_RELAXED, SC_AGENT);
              have_claim = false;
            }
            draining = true;
          }
          yield_every = __hip_atomic_load(&a.d->yield_every, __ATOMIC_RELAXED, SC_SYSTEM);
        }
        if (draining && !have_claim && waiting == 0) { action = kActExit; break; }
        // polling policy (paper Section 4.1): short back-off while spinning, longer pauses every
        // yield_every-th empty poll when the host asked for them and nothing is held
        if (yield_every != 0 && waiting == 0 && (polls % yield_every) == 0) { for (int k = 0; k < 16; ++k) __builtin_amdgcn_s_sleep(127); }
        else if (polls < 64 || waiting != 0) __builtin_amdgcn_s_sleep(1);
        else __builtin_amdgcn_s_sleep(8);
      }
      if (tid == 0) {
        s->action = action;
        s->slot = f;
        s->dep_status = dep_status;
        if (action == kActFetch) s->unit[f] = u_new;
      }
    }
    __syncthreads();
    const uint32_t action = uni(s->action), f = uni(s->slot);
    if (action == kActExit) {
      if (tid == 0) {
        uint64_t* st = a.d->stat;
        __hip_atomic_fetch_add(&st[ST_WORK_UNITS], w_units, __ATOMIC_RELAXED, SC_AGENT);
        __hip_atomic_fetch_add(&st[ST_WORK_TICKS_WAIT], w_wait, __ATOMIC_RELAXED, SC_AGENT);
        __hip_atomic_fetch_add(&st[ST_WORK_TICKS_FETCH], w_fetch, __ATOMIC_RELAXED, SC_AGENT);
        __hip_atomic_fetch_add(&st[ST_WORK_TICKS_DEP], w_dep, __ATOMIC_RELAXED, SC_AGENT);
        __hip_atomic_fetch_add(&st[ST_WORK_TICKS_EXEC], w_exec, __ATOMIC_RELAXED, SC_AGENT);
        __hip_atomic_fetch_add(&st[ST_WORK_TICKS_COMPLETE], w_done, __ATOMIC_RELAXED, SC_AGENT);
        __hip_atomic_fetch_add(&st[ST_WORK_TICKS_TOTAL], c0 - w_start, __ATOMIC_RELAXED, SC_AGENT);
      }
      return;
    }
    const uint64_t c1 = clock_if(timing || tracing);
    if (timing) { if (held_any) w_dep += c1 - c0; else w_wait += c1 - c0; }
    // the unit is the same for the whole workgroup: keep its fields in scalar registers
    const uint32_t unit_lo = uni((uint32_t)s->unit[f]), unit_hi = uni((uint32_t)(s->unit[f] >> 32));
    const uint64_t unit = ((uint64_t)unit_hi << 32) | unit_lo;
    const uint32_t chunk = (uint32_t)(unit & 0x3ffu), lap10 = (uint32_t)((unit >> 10) & 0x3ffu);
    const uint32_t slot = (uint32_t)((unit >> 20) & 0xffffu);
    const Record* r = &s->rec[f];
    if (action == kActFetch) {
      // ---- fetch the descriptor (16 lanes x 16 bytes) and the claimed table slot ----
      // The dispatcher does not wait for its mirror stores before it publishes a unit: the record is
      // taken only once its check word holds for the ticket the unit names (else its pieces are still
      // landing, or belong to the slot's previous lap) and fetched again otherwise.  The stores are on
      // their way, so this ends; it is bounded like every wait here (a workgroup that runs out leaves
      // the task to the host's time limit).
      // (the first wavefront has fetched it once already, when it saw the unit)
      bool valid = false;
      for (uint32_t attempt = 0;; ++attempt) {
        valid = mirror_record_valid(s->rec_sum, r->ticket, slot, lap10, a.cap_mask, a.cap_shift);
        if (valid || attempt >= kMirrorRetries) break;
        __syncthreads();                                  // everyone has looked at this attempt's copy
        __builtin_amdgcn_s_sleep(2);
        if (tid < 64) fetch_descriptor(a, s, rd, unit, f);
        __syncthreads();
      }
      const uint64_t c2 = clock_if(timing);
      if (timing) w_fetch += c2 - c1;
      if (!valid) {
        // never seen whole: nothing in it can be trusted, not even the ticket it would complete.  The
        // unit is dropped; the host's wait for the ticket runs into its time limit.
        __syncthreads();
        continue;
      }
      if ((r->dep[0] | r->dep[1] | r->dep[2]) != 0 && !(r->rflags & RF_DEPS_RESOLVED)) {
        // It names earlier tasks: it joins the units held, and the first wavefront looks at its done
        // words with the next poll (and runs it at once if they are all there).
        if (tid < 64) {
          waiting |= 1u << f;
          if (tid == 0) s->since[f] = wall_clock64();
        }
        continue;
      }
    }
    int32_t status = r->status;
    const uint32_t impl = uni(r->impl);
    if (status == GPUOS_OK && (s->entry[f] >> 32) != r->version) status = GPUOS_E_VERSION;
    if (status == GPUOS_OK && s->dep_status != 0) status = s->dep_status;
    const uint64_t c3 = clock_if(timing);
    // a task's start in the trace is the moment a workgroup took its descriptor (a unit that waited: when it began to)
    const uint64_t c_start = (tracing && action == kActRun) ? s->since[f] : c1;
    if (tracing && tid == 0 && chunk == 0 && r->nchunks > 1)
      __hip_atomic_store(&a.st[slot].t_first, c_start, __ATOMIC_RELAXED, SC_SYSTEM);   // in memory before this chunk is counted
    // ---- execute ----
    if (status == GPUOS_OK) status = EXEC::run(r, impl, chunk, s->red, a.progs);
    if (RING == 1 && tid == 0) __hip_atomic_fetch_add(&a.d->jit_units, 1ull, __ATOMIC_RELAXED, SC_AGENT);
    drain_stores();                   // this wave's (write-through) stores have reached memory
    __syncthreads();                  // ... and so have the other three waves'
    const uint64_t c4 = clock_if(timing || tracing);
    // ---- complete ----
    if (tid == 0) {
      const uint32_t nchunks = r->nchunks;
      bool last = true;
      if (nchunks > 1) {
        const uint32_t prev = __hip_atomic_fetch_add(&a.st[slot].chunks_done, 1u, __ATOMIC_RELAXED, SC_AGENT);
        last = (prev + 1 == nchunks);
        if (last) __hip_atomic_store(&a.st[slot].chunks_done, 0u, __ATOMIC_RELAXED, SC_SYSTEM);
      }
      if (last) {
        const uint64_t ticket = r->ticket;
        if (tracing) {
          // the tracepoint lands before the completion word that lets the host read it
          const uint64_t origin = __hip_atomic_load(&a.h->clock_origin, __ATOMIC_RELAXED, SC_SYSTEM);
          const uint64_t t_start = nchunks > 1 ? __hip_atomic_load(&a.st[slot].t_first, __ATOMIC_RELAXED, SC_SYSTEM) : c_start;
          TraceRec* tr = &a.trace[ticket & a.trace_mask];
          const uint64_t tdq = ((uint64_t)r->t_dequeue[1] << 32) | r->t_dequeue[0];
          __hip_atomic_store(&tr->t_dequeue, tdq - origin, __ATOMIC_RELAXED, SC_SYSTEM);
          __hip_atomic_store(&tr->t_start, t_start - origin, __ATOMIC_RELAXED, SC_SYSTEM);
          // The clock is read here, once this workgroup knows it finished the task: the time taken
          // right after its own chunk (c4) can lie before the start of chunk 0 when this workgroup's
          // count arrives late (seen once in a few thousand multi-chunk tasks).
          const uint64_t t_done = nchunks > 1 ? wall_clock64() : c4;
          __hip_atomic_store(&tr->t_done, t_done - origin, __ATOMIC_RELAXED, SC_SYSTEM);
          const uint64_t w4 = (uint64_t)r->version | ((uint64_t)r->op_id << 32) | ((uint64_t)(uint8_t)(int8_t)status << 48);
          __hip_atomic_store((uint64_t*)&tr->op_version, w4, __ATOMIC_RELAXED, SC_SYSTEM);
          const uint64_t w5 = (uint64_t)nchunks | ((uint64_t)blockIdx.x << 32);
          __hip_atomic_store((uint64_t*)&tr->nchunks, w5, __ATOMIC_RELAXED, SC_SYSTEM);
          __hip_atomic_store(&tr->ticket, ticket, __ATOMIC_RELAXED, SC_SYSTEM);
          drain_stores();
        }
        __hip_atomic_store(&a.st[slot].done_seq, ticket + 1, __ATOMIC_RELAXED, SC_SYSTEM);
        __hip_atomic_store(&a.hcomp[slot], pack_completion(ticket, status, r->version), __ATOMIC_RELAXED, SC_SYSTEM);
        __hip_atomic_fetch_add(&a.d->done_count, 1ull, __ATOMIC_RELAXED, SC_AGENT);
      }
    }
    __syncthreads();                  // the descriptor in LDS may be overwritten after this
    const uint64_t c5 = clock_if(timing);
    w_units += 1;
    if (timing) { w_exec += c4 - c3; w_done += c5 - c4; }
  }
}

}  // namespace gpuos
