// oracle.cpp -- CPU oracle for the GPUOS task streams.  TEST INFRASTRUCTURE ONLY:
// nothing on the product path may load this.  Single-threaded, one task after
// the other, one element after the other.  See oracle.h for what it is pinned by.
//
// What it follows:
//   * task descriptor fields: the paper's Section 4.2 submission listing
//     (operator id, input and output pointers, size) extended to the generic
//     tensor layer the abstract and Section 5.2 name (arbitrary shapes,
//     strides, dtypes, broadcasting);
//   * operator set: Section 5.2 (add, mul, ReLU, GELU; sum / max / min over a
//     small dimension) plus the ops the synthetic streams need;
//   * execution order: eager, sequential (Section 1.3).
// The paper fixes no numeric semantics; the readings used here are:
//   float math in IEEE binary32, RNE, denormals kept, no contraction except
//   the FMA op; fp16/bf16 -> fp32 exact; fp32 -> fp16/bf16 RNE, overflow to
//   inf, NaN stays NaN; transcendental ops are the mathematical function of
//   the fp32 input evaluated in double and rounded once to fp32 (mode 0);
//   every result passes through fp32 before it is rounded to the output dtype.
//
// Build: g++ -O2 -ffp-contract=off -fno-fast-math -shared -fPIC

#include "oracle.h"

#include <cmath>
#include <cstddef>
#include <cstring>
#include <limits>
#include <vector>

namespace {

inline uint32_t f2u(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }
inline float u2f(uint32_t u) { float f; std::memcpy(&f, &u, 4); return f; }

// ---- 16-bit float formats --------------------------------------------------
// binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits.
float half_to_float(uint16_t h) {
  const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
  const uint32_t e = (h >> 10) & 0x1fu;
  const uint32_t m = h & 0x3ffu;
  if (e == 0x1f) return u2f(sign | 0x7f800000u | (m << 13));          // inf / NaN
  if (e != 0) return u2f(sign | ((e + 112u) << 23) | (m << 13));      // normal
  // zero or subnormal: m * 2^-24, exact in binary32
  float v = (float)m * 5.9604644775390625e-08f;                        // 2^-24
  return (sign != 0) ? -v : v;
}

uint16_t float_to_half(float f) {
  uint32_t x = f2u(f);
  const uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
  x &= 0x7fffffffu;
  if (x > 0x7f800000u) return (uint16_t)(sign | 0x7e00u | ((x >> 13) & 0x1ffu));  // quiet NaN
  if (x >= 0x477ff000u) return (uint16_t)(sign | 0x7c00u);   // >= 65520 rounds to inf (also inf)
  const uint32_t e = x >> 23;
  if (e < 113u) {                       // result is zero or subnormal: q * 2^-24
    if (e < 102u) return sign;          // below 2^-25: rounds to zero
    const uint32_t m24 = (x & 0x7fffffu) | 0x800000u;
    const uint32_t shift = 126u - e;    // 14 .. 24
    uint32_t q = m24 >> shift;
    const uint32_t rem = m24 & ((1u << shift) - 1u);
    const uint32_t half = 1u << (shift - 1u);
    if (rem > half || (rem == half && (q & 1u))) ++q;
    return (uint16_t)(sign | q);
  }
  const uint32_t mant = x & 0x7fffffu;
  uint32_t q = ((e - 112u) << 10) | (mant >> 13);
  const uint32_t rem = mant & 0x1fffu;
  if (rem > 0x1000u || (rem == 0x1000u && (q & 1u))) ++q;     // carry may bump the exponent
  return (uint16_t)(sign | q);
}

// bfloat16: the upper 16 bits of binary32.
float bf16_to_float(uint16_t h) { return u2f((uint32_t)h << 16); }

uint16_t float_to_bf16(float f) {
  const uint32_t x = f2u(f);
  if ((x & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((x >> 16) | 0x0040u);   // quiet NaN
  const uint32_t lsb = (x >> 16) & 1u;
  return (uint16_t)((x + 0x7fffu + lsb) >> 16);
}

inline int elem_size(int dtype) { return (dtype == ORC_F32 || dtype == ORC_I32) ? 4 : 2; }
inline bool is_float(int dtype) { return dtype == ORC_F32 || dtype == ORC_F16 || dtype == ORC_BF16; }

float load_as_float(const void* base, int64_t off, int dtype) {
  switch (dtype) {
    case ORC_F32: return static_cast<const float*>(base)[off];
    case ORC_F16: return half_to_float(static_cast<const uint16_t*>(base)[off]);
    default:      return bf16_to_float(static_cast<const uint16_t*>(base)[off]);
  }
}
void store_from_float(void* base, int64_t off, int dtype, float v) {
  switch (dtype) {
    case ORC_F32: static_cast<float*>(base)[off] = v; break;
    case ORC_F16: static_cast<uint16_t*>(base)[off] = float_to_half(v); break;
    default:      static_cast<uint16_t*>(base)[off] = float_to_bf16(v); break;
  }
}

// ---- scalar operator definitions --------------------------------------------
int arity_of(int impl) {
  switch (impl) {
    case ORC_ADD: case ORC_SUB: case ORC_MUL: case ORC_DIV: case ORC_SUB_EXP: return 2;
    case ORC_FMA: return 3;
    case ORC_RELU: case ORC_EXP: case ORC_GELU_ERF: case ORC_GELU_TANH: case ORC_SCALE:
    case ORC_COPY: case ORC_SUM_LAST: case ORC_MAX_LAST: case ORC_MIN_LAST: return 1;
    case ORC_SOFTMAX_LAST: return 1;
    case ORC_MASKED_SOFTMAX_LAST: return 2;
    case ORC_LAYERNORM_LAST: return 3;
    default: return -1;
  }
}
bool is_reduction(int impl) { return impl == ORC_SUM_LAST || impl == ORC_MAX_LAST || impl == ORC_MIN_LAST; }
bool is_rowop(int impl) {
  return impl == ORC_SOFTMAX_LAST || impl == ORC_MASKED_SOFTMAX_LAST || impl == ORC_LAYERNORM_LAST;
}
bool int_capable(int impl) {
  return impl == ORC_ADD || impl == ORC_SUB || impl == ORC_MUL || impl == ORC_COPY || is_reduction(impl);
}

float exp_core(float x, int mode) {
  return mode == ORC_MODE_F64CORE ? (float)std::exp((double)x) : ::expf(x);
}

float gelu_erf(float x, int mode) {
  // x * Phi(x) written without the 1 + erf cancellation: 0.5 x erfc(-x / sqrt 2)
  if (mode == ORC_MODE_F64CORE) {
    const double xd = x;
    return (float)(0.5 * xd * std::erfc(-xd / std::sqrt(2.0)));
  }
  return 0.5f * x * ::erfcf(-x * 0.70710678118654752440f);
}

float gelu_tanh(float x, int mode) {
  // 0.5 x (1 + tanh u) == x / (1 + exp(-2u)),  u = sqrt(2/pi) (x + 0.044715 x^3)
  if (mode == ORC_MODE_F64CORE) {
    const double xd = x;
    const double u = std::sqrt(2.0 / M_PI) * (xd + 0.044715 * xd * xd * xd);
    return (float)(xd / (1.0 + std::exp(-2.0 * u)));
  }
  const float u = 0.79788456080286535588f * (x + 0.044715f * x * x * x);
  return x / (1.0f + ::expf(-2.0f * u));
}

float max_nan(float a, float b) {
  if (a != a) return a;
  if (b != b) return b;
  return a > b ? a : b;
}
float min_nan(float a, float b) {
  if (a != a) return a;
  if (b != b) return b;
  return a < b ? a : b;
}

float scalar_op(int impl, float x, float y, float z, float alpha, int mode) {
  switch (impl) {
    case ORC_ADD: return x + y;
    case ORC_SUB: return x - y;
    case ORC_MUL: return x * y;
    case ORC_DIV: return x / y;
    case ORC_RELU: return (x != x) ? x : (x > 0.0f ? x : 0.0f);
    case ORC_EXP: return exp_core(x, mode);
    case ORC_GELU_ERF: return gelu_erf(x, mode);
    case ORC_GELU_TANH: return gelu_tanh(x, mode);
    case ORC_SCALE: return x * alpha;
    case ORC_FMA: return std::fmaf(x, y, z);
    case ORC_SUB_EXP: { const float d = x - y; return exp_core(d, mode); }
    case ORC_COPY: return x;
    default: return std::numeric_limits<float>::quiet_NaN();
  }
}

// ---- descriptor checks -------------------------------------------------------
const int64_t kMaxExtent = 2147483647LL;   // sizes, numel and offsets stay below 2^31

int64_t eff_stride(const orc_tensor& t, int d) {
  return ((t.bcast_mask >> d) & 1) ? 0 : t.stride[d];
}

int check_tensor(const orc_tensor& t, int ndim, const int64_t* size, bool is_out) {
  if (t.ptr == nullptr) return ORC_E_INVAL;
  if (t.dtype > ORC_I32) return ORC_E_INVAL;
  if ((uintptr_t)t.ptr % (uintptr_t)elem_size(t.dtype) != 0) return ORC_E_INVAL;   // elements are naturally aligned
  if (is_out && t.bcast_mask != 0) return ORC_E_INVAL;
  int64_t max_off = 0;
  for (int d = 0; d < ndim; ++d) {
    if (t.stride[d] < 0) return ORC_E_INVAL;
    const int64_t s = eff_stride(t, d);
    if (is_out && size[d] > 1 && s == 0) return ORC_E_INVAL;
    if (size[d] > 1) {
      if (s > kMaxExtent) return ORC_E_INVAL;
      max_off += (size[d] - 1) * s;
      if (max_off > kMaxExtent) return ORC_E_INVAL;
    }
  }
  return ORC_OK;
}

int validate(const orc_task* t, int impl, int program_arity = 0) {
  if (impl == ORC_FAIL) return ORC_OK;            // executes nothing; reported at run time
  const int ar = program_arity > 0 ? program_arity : arity_of(impl);   // a program: elementwise, float-only, this arity
  if (ar < 0) return ORC_E_BADOP;
  if (t->ndim < 1 || t->ndim > ORC_MAX_DIMS) return ORC_E_INVAL;
  if (t->n_inputs != ar) return ORC_E_INVAL;
  int64_t numel = 1;
  for (int d = 0; d < t->ndim; ++d) {
    if (t->size[d] < 0 || t->size[d] > kMaxExtent) return ORC_E_INVAL;
    numel *= t->size[d];
    if (numel > kMaxExtent) return ORC_E_INVAL;
  }
  const bool red = is_reduction(impl);
  if (red && t->size[t->ndim - 1] == 0 && numel == 0) {
    // an empty reduced dim with a non-empty outer shape has no defined result here
    int64_t outer = 1;
    for (int d = 0; d + 1 < t->ndim; ++d) outer *= t->size[d];
    if (outer != 0) return ORC_E_INVAL;
  }
  for (int k = 0; k < ar; ++k) {
    const int rc = check_tensor(t->in[k], t->ndim, t->size, false);
    if (rc != ORC_OK) return rc;
  }
  {
    const int out_nd = red ? t->ndim - 1 : t->ndim;
    const int rc = check_tensor(t->out, out_nd, t->size, true);
    if (rc != ORC_OK) return rc;
  }
  // integer and float tensors do not mix; integer only for the ops that define it
  bool any_int = t->out.dtype == ORC_I32, all_int = t->out.dtype == ORC_I32;
  for (int k = 0; k < ar; ++k) {
    any_int = any_int || t->in[k].dtype == ORC_I32;
    all_int = all_int && t->in[k].dtype == ORC_I32;
  }
  if (any_int && !all_int) return ORC_E_INVAL;
  if (all_int && !int_capable(impl)) return ORC_E_INVAL;   // row operations are float-only (not int_capable)
  return ORC_OK;
}

// row-major linear index -> offset (elements) of operand `t`
int64_t offset_of(const orc_tensor& t, int ndim, const int64_t* size, int64_t linear) {
  int64_t off = 0;
  for (int d = 0; d < ndim; ++d) {
    int64_t inner = 1;
    for (int e = d + 1; e < ndim; ++e) inner *= size[e];
    const int64_t idx = (linear / inner) % size[d];
    off += idx * eff_stride(t, d);
  }
  return off;
}

void run_elementwise(const orc_task* t, int impl, int mode) {
  const int nd = t->ndim;
  int64_t numel = 1;
  for (int d = 0; d < nd; ++d) numel *= t->size[d];
  const bool as_int = t->out.dtype == ORC_I32;
  const bool raw_copy = impl == ORC_COPY && t->in[0].dtype == t->out.dtype;
  for (int64_t i = 0; i < numel; ++i) {
    int64_t off[3] = {0, 0, 0};
    for (int k = 0; k < t->n_inputs; ++k) off[k] = offset_of(t->in[k], nd, t->size, i);
    const int64_t oo = offset_of(t->out, nd, t->size, i);
    if (raw_copy) {
      const int es = elem_size(t->out.dtype);
      std::memcpy(static_cast<char*>(t->out.ptr) + oo * es,
                  static_cast<const char*>(t->in[0].ptr) + off[0] * es, (size_t)es);
      continue;
    }
    if (as_int) {
      const uint32_t x = static_cast<const uint32_t*>(t->in[0].ptr)[off[0]];
      const uint32_t y = t->n_inputs > 1 ? static_cast<const uint32_t*>(t->in[1].ptr)[off[1]] : 0u;
      uint32_t r = x;
      if (impl == ORC_ADD) r = x + y;
      else if (impl == ORC_SUB) r = x - y;
      else if (impl == ORC_MUL) r = x * y;
      static_cast<uint32_t*>(t->out.ptr)[oo] = r;
      continue;
    }
    float v[3] = {0.f, 0.f, 0.f};
    for (int k = 0; k < t->n_inputs; ++k) v[k] = load_as_float(t->in[k].ptr, off[k], t->in[k].dtype);
    const float r = scalar_op(impl, v[0], v[1], v[2], t->alpha, mode);
    store_from_float(t->out.ptr, oo, t->out.dtype, r);
  }
}

void run_reduction(const orc_task* t, int impl) {
  const int nd = t->ndim;
  const int ond = nd - 1;
  const int64_t n = t->size[nd - 1];
  int64_t outer = 1;
  for (int d = 0; d < ond; ++d) outer *= t->size[d];
  const int64_t s_last = eff_stride(t->in[0], nd - 1);
  for (int64_t o = 0; o < outer; ++o) {
    const int64_t in_base = offset_of(t->in[0], ond, t->size, o);
    const int64_t out_off = offset_of(t->out, ond, t->size, o);
    if (t->out.dtype == ORC_I32) {
      const int32_t* p = static_cast<const int32_t*>(t->in[0].ptr);
      uint32_t acc_sum = 0;
      int32_t acc = p[in_base];
      for (int64_t j = 0; j < n; ++j) {
        const int32_t x = p[in_base + j * s_last];
        acc_sum += (uint32_t)x;
        if (impl == ORC_MAX_LAST) acc = x > acc ? x : acc;
        if (impl == ORC_MIN_LAST) acc = x < acc ? x : acc;
      }
      static_cast<uint32_t*>(t->out.ptr)[out_off] = impl == ORC_SUM_LAST ? acc_sum : (uint32_t)acc;
      continue;
    }
    float acc = 0.0f;
    for (int64_t j = 0; j < n; ++j) {
      const float x = load_as_float(t->in[0].ptr, in_base + j * s_last, t->in[0].dtype);
      if (impl == ORC_SUM_LAST) acc = acc + x;                        // fp32, left to right
      else if (j == 0) acc = x;
      else acc = impl == ORC_MAX_LAST ? max_nan(acc, x) : min_nan(acc, x);
    }
    store_from_float(t->out.ptr, out_off, t->out.dtype, acc);
  }
}

// ---- operator programs ---------------------------------------------------------------
// One fp32 operation per instruction, in program order, on eight fp32 registers.
int validate_program(const orc_instr* code, uint32_t n, uint32_t n_inputs) {
  if (!code || n < 1 || n > ORC_PROGRAM_MAX_INSTR || n_inputs < 1 || n_inputs > 3) return ORC_E_INVAL;
  for (uint32_t i = 0; i < n; ++i)
    if (code[i].op >= ORC_PC_COUNT || code[i].dst >= ORC_PROGRAM_REGS || code[i].a >= ORC_PROGRAM_REGS ||
        code[i].b >= ORC_PROGRAM_REGS)
      return ORC_E_INVAL;
  return ORC_OK;
}

float program_value(const orc_instr* code, uint32_t n, float x, float y, float z, float alpha, int mode) {
  float r[ORC_PROGRAM_REGS] = {x, y, z, alpha, 0.f, 0.f, 0.f, 0.f};
  for (uint32_t i = 0; i < n; ++i) {
    const orc_instr& in = code[i];
    const float a = r[in.a], b = r[in.b];
    float v = 0.f;
    switch (in.op) {
      case ORC_PC_MOV: v = a; break;
      case ORC_PC_IMM: v = in.imm; break;
      case ORC_PC_ADD: v = a + b; break;
      case ORC_PC_SUB: v = a - b; break;
      case ORC_PC_MUL: v = a * b; break;
      case ORC_PC_DIV: v = a / b; break;
      case ORC_PC_FMA: v = std::fma(a, b, r[in.dst]); break;
      case ORC_PC_MAX: v = (a != a) ? a : ((b != b) ? b : (a > b ? a : b)); break;
      case ORC_PC_MIN: v = (a != a) ? a : ((b != b) ? b : (a < b ? a : b)); break;
      case ORC_PC_NEG: v = -a; break;
      case ORC_PC_ABS: v = std::fabs(a); break;
      case ORC_PC_RELU: v = (a != a) ? a : (a > 0.0f ? a : 0.0f); break;
      case ORC_PC_EXP: v = exp_core(a, mode); break;
      case ORC_PC_SQRT: v = std::sqrt(a); break;
      default: break;
    }
    r[in.dst] = v;
  }
  return r[0];
}

void run_program(const orc_task* t, const orc_instr* code, uint32_t n, int mode) {
  const int nd = t->ndim;
  int64_t numel = 1;
  for (int d = 0; d < nd; ++d) numel *= t->size[d];
  for (int64_t i = 0; i < numel; ++i) {
    float v[3] = {0.f, 0.f, 0.f};
    for (int k = 0; k < t->n_inputs; ++k)
      v[k] = load_as_float(t->in[k].ptr, offset_of(t->in[k], nd, t->size, i), t->in[k].dtype);
    store_from_float(t->out.ptr, offset_of(t->out, nd, t->size, i), t->out.dtype,
                     program_value(code, n, v[0], v[1], v[2], t->alpha, mode));
  }
}

// ---- fused row operations (Section 5.2: softmax, layer normalisation) ---------------
// Each row of the last dim is one independent problem.  The definition is the textbook one,
// evaluated in double from the inputs (fp16 / bf16 / fp32 -> double is exact); the result
// passes through fp32 and is then rounded to the output dtype, like every other result here.
//   softmax:        y_j = exp(t_j - m) / sum_k exp(t_k - m),  m = max_k t_k,
//                   t = x  or  t = alpha * x + mask (alpha widened to double, product and
//                   sum exact enough in double to count as exact);
//                   a NaN anywhere in t, a row whose maximum is +inf, or a row of all -inf
//                   gives NaN where the arithmetic above gives NaN (inf - inf);
//   layer norm:     mean = sum x / n, var = sum (x - mean)^2 / n (biased), eps = alpha,
//                   y_j = (x_j - mean) / sqrt(var + eps) * gamma_j + beta_j.
// y (nullable): unrounded doubles, row-major over the task's shape.
// store: write the rounded results into the task's output tensor.
void run_rowop(const orc_task* t, int impl, bool store, double* y_out) {
  const int nd = t->ndim, ond = nd - 1;
  const int64_t n = t->size[nd - 1];
  int64_t outer = 1;
  for (int d = 0; d < ond; ++d) outer *= t->size[d];
  if (outer == 0 || n == 0) return;
  int64_t s_last[3] = {0, 0, 0};
  for (int k = 0; k < t->n_inputs; ++k) s_last[k] = eff_stride(t->in[k], nd - 1);
  const int64_t so_last = t->out.stride[nd - 1];
  std::vector<double> v((size_t)n), res((size_t)n);
  for (int64_t o = 0; o < outer; ++o) {
    int64_t base[3] = {0, 0, 0};
    for (int k = 0; k < t->n_inputs; ++k) base[k] = offset_of(t->in[k], ond, t->size, o);
    const int64_t obase = offset_of(t->out, ond, t->size, o);
    auto in = [&](int k, int64_t j) {
      return (double)load_as_float(t->in[k].ptr, base[k] + j * s_last[k], t->in[k].dtype);
    };
    if (impl == ORC_LAYERNORM_LAST) {
      double sum = 0.0;
      for (int64_t j = 0; j < n; ++j) { v[(size_t)j] = in(0, j); sum += v[(size_t)j]; }
      const double mean = sum / (double)n;
      double ss = 0.0;
      for (int64_t j = 0; j < n; ++j) {
        const double d = v[(size_t)j] - mean;
        ss += d * d;
      }
      const double var = ss / (double)n;
      const double rstd = 1.0 / std::sqrt(var + (double)t->alpha);
      for (int64_t j = 0; j < n; ++j) {
        const double g = in(1, j), b = in(2, j);
        res[(size_t)j] = (v[(size_t)j] - mean) * rstd * g + b;
      }
    } else {
      bool any_nan = false;
      double m = -HUGE_VAL;
      for (int64_t j = 0; j < n; ++j) {
        double a = in(0, j);
        if (impl == ORC_MASKED_SOFTMAX_LAST) a = (double)t->alpha * a + in(1, j);
        v[(size_t)j] = a;
        if (a != a) any_nan = true;
        else if (a > m) m = a;
      }
      double sum = 0.0;
      for (int64_t j = 0; j < n; ++j) { res[(size_t)j] = std::exp(v[(size_t)j] - m); sum += res[(size_t)j]; }
      for (int64_t j = 0; j < n; ++j) res[(size_t)j] = any_nan ? std::nan("") : res[(size_t)j] / sum;
    }
    for (int64_t j = 0; j < n; ++j) {
      if (y_out) y_out[o * n + j] = res[(size_t)j];
      if (store) store_from_float(t->out.ptr, obase + j * so_last, t->out.dtype, (float)res[(size_t)j]);
    }
  }
}

}  // namespace

extern "C" {

int orc_validate(const orc_task* t, int impl) { return validate(t, impl); }

int orc_run_task(const orc_task* t, int impl, int mode) {
  const int rc = validate(t, impl);
  if (rc != ORC_OK) return rc;
  if (impl == ORC_FAIL) return ORC_E_BADOP;
  if (is_reduction(impl)) run_reduction(t, impl);
  else if (is_rowop(impl)) run_rowop(t, impl, true, nullptr);
  else run_elementwise(t, impl, mode);
  return ORC_OK;
}

int64_t orc_run_stream(const orc_task* tasks, int64_t n, const int32_t* impl, int mode,
                       int32_t* status) {
  int64_t bad = 0;
  for (int64_t i = 0; i < n; ++i) {
    const int rc = orc_run_task(&tasks[i], impl[i], mode);
    if (status) status[i] = rc;
    if (rc != ORC_OK) ++bad;
  }
  return bad;
}

int orc_sum_last_f64(const orc_task* t, double* sum, double* l1) {
  const int rc = validate(t, ORC_SUM_LAST);
  if (rc != ORC_OK) return rc;
  if (!is_float(t->in[0].dtype)) return ORC_E_INVAL;
  const int nd = t->ndim, ond = nd - 1;
  const int64_t n = t->size[nd - 1];
  int64_t outer = 1;
  for (int d = 0; d < ond; ++d) outer *= t->size[d];
  const int64_t s_last = eff_stride(t->in[0], nd - 1);
  for (int64_t o = 0; o < outer; ++o) {
    const int64_t in_base = offset_of(t->in[0], ond, t->size, o);
    double s = 0.0, a = 0.0;
    for (int64_t j = 0; j < n; ++j) {
      const double x = load_as_float(t->in[0].ptr, in_base + j * s_last, t->in[0].dtype);
      s += x;
      a += std::fabs(x);
    }
    sum[o] = s;
    l1[o] = a;
  }
  return ORC_OK;
}

int orc_validate_program(const orc_instr* code, uint32_t n_instr, uint32_t n_inputs) {
  return validate_program(code, n_instr, n_inputs);
}

int orc_run_task_program(const orc_task* t, const orc_instr* code, uint32_t n_instr, uint32_t n_inputs, int mode) {
  int rc = validate_program(code, n_instr, n_inputs);
  if (rc != ORC_OK) return rc;
  rc = validate(t, ORC_COPY, (int)n_inputs);        // the rules of an elementwise operator of this arity ...
  if (rc != ORC_OK) return rc;
  if (t->out.dtype == ORC_I32) return ORC_E_INVAL;  // ... but programs are float-only
  run_program(t, code, n_instr, mode);
  return ORC_OK;
}

int orc_rowop_f64(const orc_task* t, int impl, double* y) {
  if (!is_rowop(impl)) return ORC_E_INVAL;
  const int rc = validate(t, impl);
  if (rc != ORC_OK) return rc;
  run_rowop(t, impl, false, y);
  return ORC_OK;
}

float orc_f16_to_f32(uint16_t h) { return half_to_float(h); }
uint16_t orc_f32_to_f16(float f) { return float_to_half(f); }
float orc_bf16_to_f32(uint16_t h) { return bf16_to_float(h); }
uint16_t orc_f32_to_bf16(float f) { return float_to_bf16(f); }
float orc_scalar_op(int impl, float x, float y, float z, float alpha, int mode) {
  return scalar_op(impl, x, y, z, alpha, mode);
}

void orc_abi_layout(uint32_t out[8]) {
  out[0] = (uint32_t)sizeof(orc_task);
  out[1] = (uint32_t)sizeof(orc_tensor);
  out[2] = (uint32_t)offsetof(orc_task, size);
  out[3] = (uint32_t)offsetof(orc_task, in);
  out[4] = (uint32_t)offsetof(orc_task, out);
  out[5] = (uint32_t)offsetof(orc_task, alpha);
  out[6] = (uint32_t)offsetof(orc_task, dep);
  out[7] = 32u;
}

}  // extern "C"
