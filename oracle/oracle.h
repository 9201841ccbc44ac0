/*
 * oracle.h -- CPU oracle for the GPUOS task streams.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-threaded executor of the same task descriptors the
 * GPU library takes: tasks are run one after the other in ticket order, each
 * to completion (the eager-execution semantics the paper's Section 1.3 says
 * the method retains).  No queue, no table, no chunking, no contiguity or
 * coalescing shortcuts: every element is reached through the row-major
 * index -> per-dim index -> strided offset definition.
 *
 * It shares no code with the HIP path.  The two struct layouts below repeat
 * the GPU library's descriptor layout on purpose (the interface has to be the
 * same for the same seeded task arrays to drive both); the tests compare the
 * two layouts through orc_abi_layout().
 *
 * Only tests/, the smoke check and the benchmark's cpu_baseline leg may load
 * this library.  Parity status: every function here is pinned by CPU tests
 * (hand values, numpy strided views, exhaustive 16-bit conversions, closed
 * forms); nothing is "parity unpinned".
 */
#ifndef GPUOS_ORACLE_H_
#define GPUOS_ORACLE_H_
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

enum { ORC_MAX_DIMS = 6 };
enum { ORC_F32 = 0, ORC_F16 = 1, ORC_BF16 = 2, ORC_I32 = 3 };
enum {
  ORC_ADD = 1, ORC_SUB = 2, ORC_MUL = 3, ORC_DIV = 4, ORC_RELU = 5, ORC_EXP = 6,
  ORC_GELU_ERF = 7, ORC_GELU_TANH = 8, ORC_SCALE = 9, ORC_FMA = 10,
  ORC_SUB_EXP = 11, ORC_COPY = 12, ORC_SUM_LAST = 13, ORC_MAX_LAST = 14,
  ORC_MIN_LAST = 15, ORC_FAIL = 16,
  /* fused row operations (Section 5.2 lists softmax and layer normalisation) */
  ORC_SOFTMAX_LAST = 17,         /* y = softmax over the last dim of x                      */
  ORC_MASKED_SOFTMAX_LAST = 18,  /* y = softmax over the last dim of alpha * x + mask       */
  ORC_LAYERNORM_LAST = 19        /* y = (x - mean) / sqrt(var + alpha) * gamma + beta,
                                    mean and (biased) variance over the last dim            */
};
enum { ORC_OK = 0, ORC_E_INVAL = -1, ORC_E_BADOP = -3 };
enum { ORC_FLAG_FENCE = 1, ORC_FLAG_KEEPDIM = 2 };

/* transcendental cores: 0 = evaluate in double from the fp32 input, round once
 * to fp32 (the definition the GPU is gated against); 1 = glibc fp32 routines */
enum { ORC_MODE_F64CORE = 0, ORC_MODE_F32LIBM = 1 };

typedef struct orc_tensor {
  void*   ptr;                  /* HOST address of element 0 */
  int64_t stride[ORC_MAX_DIMS]; /* elements */
  uint8_t dtype;
  uint8_t bcast_mask;
  uint8_t reserved[6];
} orc_tensor;

typedef struct orc_task {
  uint16_t op_id;
  uint8_t  ndim;
  uint8_t  n_inputs;
  uint32_t flags;
  int64_t  size[ORC_MAX_DIMS];
  orc_tensor in[3];
  orc_tensor out;
  float    alpha;
  uint16_t dep[3];
  uint16_t reserved[3];
} orc_task;

/* Validate one descriptor against `impl` (same host-detectable rules as the
 * library's submit).  Returns ORC_OK / ORC_E_INVAL / ORC_E_BADOP. */
int orc_validate(const orc_task* t, int impl);

/* Execute one task with implementation `impl`.  FAIL writes nothing and
 * returns ORC_E_BADOP. */
int orc_run_task(const orc_task* t, int impl, int mode);

/* Execute tasks[0..n) in order.  impl[i] is the implementation of task i (the
 * harness resolves logical op + recorded version -> impl).  status (nullable)
 * receives the per-task result.  Returns the number of tasks whose status is
 * not ORC_OK. */
int64_t orc_run_stream(const orc_task* tasks, int64_t n, const int32_t* impl,
                       int mode, int32_t* status);

/* For a SUM_LAST task: per output row, the sum accumulated in double and the
 * L1 norm of the row (inputs converted to fp32 first).  Both arrays have one
 * entry per outer index in row-major order.  Used for the reduction
 * tolerance |g - o| <= 1e-5 * max(|o|, L1/sqrt(n)). */
int orc_sum_last_f64(const orc_task* t, double* sum, double* l1);

/* For a row operation (softmax, masked softmax, layer norm): the results
 * BEFORE any rounding, evaluated in double from the inputs (each converted
 * exactly to double), one value per element in row-major order of the task's
 * shape.  (The error bound a float32 evaluation is held to is derived by the
 * tests from these values and the inputs; it is no output of the oracle.) */
int orc_rowop_f64(const orc_task* t, int impl, double* y);

/* Operator programs: an elementwise operator given as a short list of
 * instructions instead of a built-in id (the role of the paper's runtime
 * operator injection, Sections 1.2 and 4.1).  Eight fp32 registers; on entry
 * r0, r1, r2 hold the inputs converted to fp32 (0 for inputs the task does not
 * have), r3 = alpha, r4..r7 = 0.  Each instruction is ONE IEEE binary32
 * operation (RNE, denormals kept) on registers: dst = op(a, b):
 *   MOV a | IMM imm | ADD | SUB | MUL | DIV | FMA fma(a, b, dst) (one rounding) |
 *   MAX, MIN (a NaN operand wins, a first; else a > b ? a : b resp. a < b ? a : b) |
 *   NEG | ABS | RELU (a > 0 ? a : +0, NaN stays) | EXP (the mathematical
 *   function, evaluated per `mode` like the EXP operator) | SQRT (correctly rounded).
 * The result is r0 after the last instruction, rounded to the output dtype. */
enum {
  ORC_PC_MOV = 0, ORC_PC_IMM = 1, ORC_PC_ADD = 2, ORC_PC_SUB = 3, ORC_PC_MUL = 4, ORC_PC_DIV = 5,
  ORC_PC_FMA = 6, ORC_PC_MAX = 7, ORC_PC_MIN = 8, ORC_PC_NEG = 9, ORC_PC_ABS = 10, ORC_PC_RELU = 11,
  ORC_PC_EXP = 12, ORC_PC_SQRT = 13, ORC_PC_COUNT = 14
};
typedef struct orc_instr { uint8_t op, dst, a, b; float imm; } orc_instr;   /* 8 bytes */
enum { ORC_PROGRAM_MAX_INSTR = 32, ORC_PROGRAM_REGS = 8 };

/* ORC_OK if the program is well-formed (1..32 instructions, 1..3 inputs, known
 * opcodes, register numbers below 8), else ORC_E_INVAL. */
int orc_validate_program(const orc_instr* code, uint32_t n_instr, uint32_t n_inputs);

/* Execute one elementwise task whose operator is the program (task.n_inputs
 * must equal n_inputs; float tensors only; descriptor rules as orc_validate
 * for an elementwise operator of that arity). */
int orc_run_task_program(const orc_task* t, const orc_instr* code, uint32_t n_instr, uint32_t n_inputs, int mode);

/* scalar conversions, exported so the tests can sweep all 65536 patterns */
float    orc_f16_to_f32(uint16_t h);
uint16_t orc_f32_to_f16(float f);
float    orc_bf16_to_f32(uint16_t h);
uint16_t orc_f32_to_bf16(float f);
/* one elementwise result in fp32 (before rounding to the output dtype) */
float    orc_scalar_op(int impl, float x, float y, float z, float alpha, int mode);

void orc_abi_layout(uint32_t out[8]);

#ifdef __cplusplus
}
#endif
#endif
