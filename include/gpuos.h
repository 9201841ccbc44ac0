/*
 * gpuos.h -- C ABI of the MI355X-native GPUOS hot path.
 *
 * One long-lived ("persistent") HIP worker kernel drains a host-fed ring of
 * task descriptors and executes small tensor operations (elementwise ops,
 * last-dim reductions and fused row operations over <=6-D strided / broadcast
 * tensors, and operators defined at run time as short programs) through a
 * versioned dual-slot operator table.  The design follows the paper's
 * Section 4.1 (ring buffer channel, persistent kernel executor, dynamic
 * operator table), Section 4.2 (task submission protocol: acquire slot,
 * write, commit with a store-release; device poll with a load-acquire) and
 * Section 5.4 / Table 1 (host runtime calls init, fuse, set_yield_every,
 * peek_queue, worker_alive, shutdown).
 *
 * Conventions that hold for every call below
 *   - plain C types only; `void*` tensor pointers are DEVICE pointers that the
 *     caller owns (allocated beforehand, paper Section 4.3) and keeps alive
 *     and unmodified until gpuos_wait() has covered the ticket;
 *   - every call returns 0 (GPUOS_OK) or a negative gpuos_status; nothing
 *     throws or aborts across this boundary;
 *   - any number of host threads may call gpuos_submit / gpuos_submit_flush / gpuos_flush /
 *     gpuos_wait / gpuos_register_op / gpuos_swap_op / the query calls on one
 *     context at the same time (Section 6.4 speaks of many concurrent host
 *     threads on one ring): descriptors are validated and packed in
 *     the calling thread, ticket reservation and the ring writes are
 *     serialised inside the library, so the tickets of one gpuos_submit call
 *     are consecutive and dependencies (back-distances) inside that call mean
 *     what they say; a back-distance that reaches before the call's first
 *     ticket names whatever another thread may have enqueued there, so only
 *     a single producer may use those.  gpuos_init / gpuos_shutdown /
 *     gpuos_stop_worker / gpuos_start_worker are for one thread;
 *   - while a context is alive the worker kernel is resident on its own
 *     non-blocking stream: the caller must not call hipDeviceSynchronize(),
 *     hipFree() or anything else that waits for "all streams" before
 *     gpuos_shutdown(), or the process deadlocks.  Other kernels share the
 *     compute units with the worker: it is built for 128 vector registers per
 *     lane and the default of 3 workgroups per compute unit leaves a quarter of
 *     every register file, and more than half of the local memory and wave
 *     slots, to them.  With workgroups_per_cu = 4 the worker fills every
 *     register file and NO other kernel can start until it exits -- that
 *     includes the copy kernel the HIP runtime uses for device<->host copies of
 *     16 KiB or less (larger ones go to the DMA engines): use 4 only for a
 *     process that runs nothing else on the GPU, and then move small results
 *     with a GPUOS_IMPL_COPY task into pinned, device-mapped host memory or
 *     read them after gpuos_stop_worker().  Kernels that need more registers
 *     or local memory than the worker leaves (large matrix products do, even at
 *     3 and 2 workgroups per compute unit) wait until it has left: hand them
 *     the GPU with gpuos_stop_worker() ... gpuos_start_worker(), or let
 *     cfg.idle_exit_ms do so.
 */
#ifndef GPUOS_H_
#define GPUOS_H_

#if !defined(__HIPCC_RTC__)
#include <stdint.h>
#endif

#ifdef __cplusplus
extern "C" {
#endif

#define GPUOS_MAX_DIMS   6      /* generic tensor descriptor: up to 6 dims        */
#define GPUOS_MAX_INPUTS 3
#define GPUOS_MAX_OPS    256    /* logical operator ids are 0 .. 255              */
#define GPUOS_ALL        (~0ull)/* gpuos_wait: every ticket submitted so far      */

typedef struct gpuos_ctx gpuos_ctx;   /* opaque; owned by the library */

/* ---- status codes ------------------------------------------------------ */
enum gpuos_status {
  GPUOS_OK        =  0,
  GPUOS_E_INVAL   = -1,   /* malformed argument or descriptor                     */
  GPUOS_E_FULL    = -2,   /* non-blocking submit: not enough free ring slots      */
  GPUOS_E_BADOP   = -3,   /* unknown / unregistered / failed operator             */
  GPUOS_E_TIMEOUT = -4,   /* a bounded wait ran out                               */
  GPUOS_E_DEAD    = -5,   /* worker kernel is not running (shutdown / watchdog)   */
  GPUOS_E_HIP     = -6,   /* a HIP runtime call failed (see gpuos_last_hip_error) */
  GPUOS_E_NOMEM   = -7,
  GPUOS_E_VERSION = -8    /* device found a table entry whose version differs from
                             the one the task claimed (protocol violation)        */
};

/* ---- element types ------------------------------------------------------ */
enum gpuos_dtype { GPUOS_F32 = 0, GPUOS_F16 = 1, GPUOS_BF16 = 2, GPUOS_I32 = 3 };

/* ---- built-in device implementations an operator-table entry can name -----
 * (operator library, paper Section 5.2: elementwise add / mul / ReLU / GELU and
 * sum / max / min reductions, plus what the task streams need).  x, y, z are
 * the inputs converted to fp32, a = task.alpha.  All float math is IEEE
 * binary32 round-to-nearest-even with denormals kept; the result is rounded
 * once more to the output dtype.  EXP / GELU are the mathematical functions
 * (the device evaluates them so that the fp32 result is within 2 ulp).
 *   ADD x+y  SUB x-y  MUL x*y  DIV x/y  RELU (x>0 ? x : +0, NaN->NaN)
 *   EXP e^x  GELU_ERF 0.5 x erfc(-x/sqrt 2)  GELU_TANH x/(1+e^(-2u)),
 *   u = sqrt(2/pi)(x+0.044715 x^3)  SCALE x*a  FMA fma(x,y,z)
 *   SUB_EXP e^(fl32(x-y))  COPY x (bit copy when dtypes match)
 *   SUM_LAST / MAX_LAST / MIN_LAST reduce the last dim (fp32 accumulator for
 *   floats, two's-complement wrap for I32; max/min propagate NaN)
 *   FAIL: kill-switch stub (paper Section 5.3): completes at once with
 *   status GPUOS_E_BADOP and writes nothing.
 * Fused row operations (Section 5.2 names softmax and layer normalisation):
 * every row of the last dim is one problem, the output has the input's shape,
 * further inputs broadcast like any other operand.  Defined as the exact
 * function of the inputs; the device evaluates in fp32 (row held in
 * registers, one read and one write of the row) to within
 * 2^-22 * (the magnitude its rounding errors scale with) of it, then rounds
 * to the output dtype.  Float tensors only.
 *   SOFTMAX_LAST (x): y_j = e^(x_j - m) / sum_k e^(x_k - m), m = max_k x_k
 *   MASKED_SOFTMAX_LAST (x, mask): the same on t = a * x + mask
 *     (mask entries of -inf give exactly 0; a row with a NaN, a +inf or
 *     nothing but -inf is all NaN)
 *   LAYERNORM_LAST (x, gamma, beta): (x - mean) / sqrt(var + a) * gamma + beta
 *     with the mean and the biased variance of the row, a = epsilon.
 * I32 tensors are accepted by ADD SUB MUL COPY SUM_LAST MAX_LAST MIN_LAST only,
 * and only when every tensor of the task is I32. */
enum gpuos_impl {
  GPUOS_IMPL_NONE = 0,
  GPUOS_IMPL_ADD = 1, GPUOS_IMPL_SUB = 2, GPUOS_IMPL_MUL = 3, GPUOS_IMPL_DIV = 4,
  GPUOS_IMPL_RELU = 5, GPUOS_IMPL_EXP = 6, GPUOS_IMPL_GELU_ERF = 7,
  GPUOS_IMPL_GELU_TANH = 8, GPUOS_IMPL_SCALE = 9, GPUOS_IMPL_FMA = 10,
  GPUOS_IMPL_SUB_EXP = 11, GPUOS_IMPL_COPY = 12,
  GPUOS_IMPL_SUM_LAST = 13, GPUOS_IMPL_MAX_LAST = 14, GPUOS_IMPL_MIN_LAST = 15,
  GPUOS_IMPL_FAIL = 16,
  GPUOS_IMPL_SOFTMAX_LAST = 17, GPUOS_IMPL_MASKED_SOFTMAX_LAST = 18,
  GPUOS_IMPL_LAYERNORM_LAST = 19,
  GPUOS_IMPL_COUNT = 20
};

/* ---- operator programs: operators defined while the worker runs ----------
 * The paper injects new operators into the running kernel by compiling device
 * code at run time and publishing its address through the dual-slot table
 * (Sections 1.2, 4.1).  Here a new ELEMENTWISE operator is given as a short
 * program.  The resident kernel can interpret it, and the library compiles it
 * at run time into native code that a second resident kernel executes (see
 * gpuos_native_info below); a kernel that is already running cannot call into
 * a code object loaded later, hence the second kernel.  The rest of the
 * protocol is the paper's: gpuos_define_program stores the program in a
 * device-visible table and returns an implementation id; gpuos_register_op /
 * gpuos_swap_op bind a logical operator to it through the inactive slot and
 * the version flip, without stopping the worker.
 * Eight fp32 registers.  On entry r0, r1, r2 = the task's inputs converted to
 * fp32 (0 where the task has fewer), r3 = task.alpha, r4..r7 = 0.  Every
 * instruction is ONE IEEE binary32 operation (RNE, denormals kept),
 * dst = op(a, b); the result is r0 after the last instruction, rounded to the
 * output dtype.  Float tensors only; any shapes, strides, dtypes, broadcast. */
enum gpuos_opcode {
  GPUOS_PC_MOV = 0,   /* dst = a                                               */
  GPUOS_PC_IMM = 1,   /* dst = imm                                             */
  GPUOS_PC_ADD = 2, GPUOS_PC_SUB = 3, GPUOS_PC_MUL = 4, GPUOS_PC_DIV = 5,
  GPUOS_PC_FMA = 6,   /* dst = fma(a, b, dst), one rounding                    */
  GPUOS_PC_MAX = 7, GPUOS_PC_MIN = 8,  /* a NaN operand wins (a first); else a > b ? a : b,
                                          resp. a < b ? a : b                  */
  GPUOS_PC_NEG = 9, GPUOS_PC_ABS = 10,
  GPUOS_PC_RELU = 11, /* a > 0 ? a : +0, NaN stays NaN                         */
  GPUOS_PC_EXP = 12,  /* e^a, within 2 ulp like GPUOS_IMPL_EXP                 */
  GPUOS_PC_SQRT = 13, /* correctly rounded                                     */
  GPUOS_PC_COUNT = 14
};
typedef struct gpuos_instr {
  uint8_t op, dst, a, b;            /* enum gpuos_opcode; register numbers 0..7   */
  float   imm;                      /* GPUOS_PC_IMM only                          */
} gpuos_instr;                      /* 8 bytes */
#define GPUOS_PROGRAM_MAX_INSTR 32
#define GPUOS_PROGRAM_REGS      8
#define GPUOS_MAX_PROGRAMS      64
#define GPUOS_IMPL_PROGRAM_BASE 64  /* implementation ids 64 .. 127 name programs */

/* Native code for programs.  Interpreting costs time per element (a six-instruction program runs
 * at well under half the speed of a built-in), so unless cfg.jit_mode says otherwise every
 * gpuos_define_program also compiles, with the HIP run-time compiler, a SECOND resident worker
 * kernel that holds all programs defined so far as straight-line native functors inside the
 * library's own elementwise execution paths (same arithmetic, instruction by instruction, as the
 * interpreter).  The dispatcher then routes the tasks of those programs to that kernel's work-unit
 * ring; table, versions, dependencies and completions are shared with the worker, which never
 * stops.  The kernel is built when an operator is first bound (gpuos_register_op / gpuos_swap_op)
 * to a program that is not native yet, for all programs defined by then (cfg.jit_mode = 1: at
 * every gpuos_define_program): that call compiles in the calling thread (one to two seconds; code
 * objects are cached per process by the hash of the generated source), lets the previous
 * generation of the kernel drain and leave, launches the new one, and only then binds.  Until
 * then, and whenever this path is unavailable or fails, programs are interpreted.
 * gpuos_native_info: out[0] 1 when programs are being served as native code, out[1] generation of
 * the run-time kernel, out[2] programs it holds, out[3] kernels compiled by this context, out[4]
 * taken from the cache, out[5] work units it has executed (valid after gpuos_stop_worker, else
 * 0), out[6] microseconds the last compilation took, out[7] its workgroups; why (nullable, HOST
 * buffer of why_len bytes): the reason when the native path is off or was given up. */
int gpuos_native_info(gpuos_ctx* ctx, uint64_t out[8], char* why, uint32_t why_len);

/* ---- task flags --------------------------------------------------------- */
#define GPUOS_FLAG_FENCE   1u  /* start only after EVERY earlier ticket completed  */
#define GPUOS_FLAG_KEEPDIM 2u  /* reductions: output keeps a trailing dim of size 1
                                  (its stride is ignored)                          */

/* ---- generic tensor descriptor (paper abstract / Section 5.2: arbitrary
 * shapes, strides, dtypes and broadcasting) -------------------------------- */
typedef struct gpuos_tensor {
  void*   ptr;                      /* device address of the element at index 0, a
                                     * multiple of the element size (else E_INVAL)   */
  int64_t stride[GPUOS_MAX_DIMS];   /* in ELEMENTS, >= 0; entries >= ndim ignored   */
  uint8_t dtype;                    /* enum gpuos_dtype                             */
  uint8_t bcast_mask;               /* bit d set: dim d is broadcast (stride := 0)  */
  uint8_t reserved[6];
} gpuos_tensor;                     /* 64 bytes */

/* ---- task descriptor as the caller fills it (paper Section 4.2 listing:
 * op id, input / output pointers, size; extended to the generic tensor layer).
 * gpuos_submit validates it, coalesces dims and packs it into a fixed 256-byte
 * ring record; the caller's copy is not referenced after submit returns. ----- */
typedef struct gpuos_task {
  uint16_t op_id;                   /* logical operator id (index into the table)   */
  uint8_t  ndim;                    /* 1 .. 6                                       */
  uint8_t  n_inputs;                /* must equal the arity of the op's impl        */
  uint32_t flags;                   /* GPUOS_FLAG_*                                 */
  int64_t  size[GPUOS_MAX_DIMS];    /* elementwise: iteration (= output) shape;
                                       reductions: the INPUT shape, the last dim is
                                       reduced, output shape = size[0 .. ndim-2]    */
  gpuos_tensor in[GPUOS_MAX_INPUTS];
  gpuos_tensor out;
  float    alpha;                   /* SCALE multiplier                             */
  uint16_t dep[3];                  /* 0 = none; k = wait for ticket (mine - k)     */
  uint16_t reserved[3];
} gpuos_task;                       /* 328 bytes */

/* per-ticket completion record (paper Section 5.3 tracepoint fields: task id,
 * operator-table version; timestamps are host steady_clock nanoseconds) */
typedef struct gpuos_completion {
  uint64_t ticket;
  int32_t  status;                  /* gpuos_status reported by the device          */
  uint32_t op_version;              /* table version the task claimed               */
  uint64_t t_submit_ns;             /* doorbell time of the batch that published it */
  uint64_t t_done_ns;               /* time the host first saw the completion word  */
} gpuos_completion;                 /* 32 bytes */

/* Device-side tracepoint of one task (paper Section 5.3: task id, dequeue
 * time, execution time, operator-table version), written by the workgroup that
 * finishes the task into a ring in host memory that can be read while the
 * worker runs.  Times are ticks of the device's constant 100 MHz clock (10 ns)
 * since the worker kernel started. */
typedef struct gpuos_trace_record {
  uint64_t ticket;
  uint64_t t_dequeue;               /* dispatcher took the task from the ring          */
  uint64_t t_start;                 /* the workgroup that ran chunk 0 had claimed it   */
  uint64_t t_done;                  /* the last chunk's stores had reached memory      */
  uint32_t op_version;              /* table version the task claimed                  */
  uint16_t op_id;
  int8_t   status;
  uint8_t  reserved;
  uint32_t nchunks;                 /* work units the task was split into              */
  uint32_t workgroup;               /* workgroup that ran the last chunk               */
} gpuos_trace_record;               /* 48 bytes */

/* paper Table 1 peek_queue(): head, tail, processed counts */
typedef struct gpuos_queue_state {
  uint64_t head_submitted;          /* tickets written into the ring by the host    */
  uint64_t tail_published;          /* tickets made visible by the last doorbell    */
  uint64_t claimed;                 /* tickets the device has dequeued from the ring*/
  uint64_t completed;               /* completed-in-order floor seen by the host    */
  uint64_t heartbeat;               /* worker poll-loop counter (liveness)          */
  uint32_t capacity;
  uint32_t workgroups;              /* resident worker workgroups                   */
  uint32_t push_ring;               /* 1: the ring lives in device memory (cfg.push_ring
                                       as resolved at init)                          */
  uint32_t reserved;
} gpuos_queue_state;

typedef struct gpuos_config {
  int32_t  device;                  /* HIP device ordinal                           */
  uint32_t threads_per_workgroup;   /* paper's threads_per_block; 0 => 256 (only 256
                                       is supported by the built kernel)            */
  uint32_t workgroups_per_cu;       /* 0 => 3; 1..4, clamped to what is co-resident; 4 leaves no room for other kernels (see above) */
  uint32_t nonblocking_submit;      /* 1: a full ring returns GPUOS_E_FULL          */
  uint32_t harvester_thread;        /* 1: a pinned host thread harvests completions
                                       and time-stamps them (latency measurement)   */
  uint32_t defer_op_check;          /* 1: do not reject unknown op ids at submit;
                                       the device bounds-checks and reports them    */
  uint32_t idle_exit_ms;            /* worker exits by itself after this long with
                                       an empty ring (0 = never, the paper's mode)  */
  uint32_t wait_timeout_ms;         /* bound on every internal blocking wait
                                       (0 => 30000)                                 */
  uint32_t completion_log;          /* tickets kept for gpuos_get_completions
                                       (0 => 1<<21; rounded up to a power of two)   */
  uint32_t chunk_elems;             /* elements of a large task one workgroup takes at a time,
                                       quoted for 12 bytes of traffic per element and scaled for
                                       other operators (0 => 16384; rounded up to a multiple of
                                       1024).  Tasks of up to 2^20 elements and links of a chain
                                       take half of it; a task of at most four such chunks is cut
                                       into up to four; gathered and transposed inputs are spread
                                       over up to 32 resp. 64 workgroups (gpuos_task_plan tells) */
  uint32_t push_ring;               /* where the ring, the doorbell and the table source
                                       live: 0 = fine-grained host memory that the device
                                       polls over PCIe; 1 = device memory that the host
                                       writes through the PCIe BAR (needs a host-visible
                                       BAR; the device then polls its own memory and a
                                       dispatcher pass is about half as long); 2 = 1 when
                                       the device reports a large BAR, else 0 (default)   */
  uint32_t trace_entries;           /* > 0: keep a device-written trace record for the
                                       last this-many tickets (rounded up to a power of
                                       two, at most 1<<20) and count dispatched tasks per
                                       operator; 0: tracing off (default)               */
  uint32_t markers;                 /* 1: annotate the host calls for a profiler's marker
                                       trace (rocprofv3 --marker-trace): ranges around
                                       gpuos_submit and gpuos_wait, marks at init, table
                                       changes, stop and start.  The roctx library is
                                       looked up at run time (the environment variable
                                       GPUOS_ROCTX_LIBRARY names another one); without it
                                       the option does nothing.  0: off (default)          */
  uint32_t phase_timers;            /* 1: the dispatcher and the workers time every phase of
                                       their work for gpuos_worker_stats (about a dozen reads
                                       of the device clock per task: measurable on small
                                       tasks); 0: only the counts are kept (default)        */
  uint32_t dep_wait_us;             /* bound, in microseconds, on the time a worker workgroup waits
                                       for a dependency of the task it holds (what it waits for was
                                       published before its own unit, so the wait ends by itself; the
                                       bound is a safety net).  A task that runs into it completes
                                       with GPUOS_E_TIMEOUT and writes nothing; its dependants run.
                                       0 => wait_timeout_ms                                    */
  uint32_t jit_mode;                /* operators defined as programs (gpuos_define_program): 0 => they
                                       are also compiled to native code at run time and served by a
                                       second resident worker kernel, built when an operator is first
                                       bound to a program that is not native yet (needs the HIP
                                       run-time compiler library; without it, or when anything in that
                                       path fails, they stay interpreted); 1 => the same, built at
                                       every gpuos_define_program; 2 => interpreted only            */
  uint32_t jit_workgroups_per_cu;   /* workgroups per compute unit of that second kernel.  0 => 1 if
                                       that leaves a workgroup's place per compute unit free for other
                                       kernels (the HIP runtime's copy kernels included), else none:
                                       on MI355X four workgroups fit a compute unit, so programs run
                                       natively by default with workgroups_per_cu <= 2 and are
                                       interpreted beside the default 3.  A number given here is taken
                                       as it is (clamped to what is co-resident): 3 + 1 fills every
                                       register file, and nothing else starts on the GPU until a
                                       worker leaves (gpuos_native_info says which case holds)        */
  uint32_t reserved[1];
} gpuos_config;

/* Fill *cfg with the defaults named above. */
void gpuos_default_config(gpuos_config* cfg);

/* Paper Table 1 init(capacity, threads_per_block): allocate the ring (host
 * memory, fine-grained coherent, mapped to the device), the device-side mirror
 * and operator table, and launch the persistent worker once.
 * queue_capacity: power of two in [2, 65536]; 0 => 4096 (the paper's default).
 * cfg: NULL => defaults on the current device.  *out receives the context. */
int gpuos_init(gpuos_ctx** out, uint32_t queue_capacity, const gpuos_config* cfg);

/* gpuos_init for callers that cannot allocate (harnesses that forbid hipMalloc /
 * hipHostMalloc at run time, serving loops that set a context up and tear it down
 * over and over): the same context and the same worker kernel, but the call
 * allocates nothing, neither on the device nor on the host.  The device-side state
 * (control block, ring mirror, work-unit ring, done words, operator table) lives in
 * a file-scope device array of the library, about 8.3 MiB that every GPU the library
 * is loaded on holds until the process ends; everything the host side needs (the
 * context object, ring, doorbell, completion words and log, table source, programs)
 * lives in host_block.
 *   queue_capacity: power of two in [2, GPUOS_STATIC_MAX_CAPACITY]; 0 => the maximum.
 *     A larger value is GPUOS_E_INVAL (gpuos_last_hip_error() says why).
 *   cfg: as for gpuos_init (NULL => defaults); push_ring is ignored (the ring is
 *     in host_block, polled by the device); harvester_thread and trace_entries must
 *     be 0 (they allocate); completion_log is queue_capacity.
 *   host_block: caller-owned HOST memory that the device can read and write
 *     coherently (hipHostMalloc with hipHostMallocCoherent | hipHostMallocMapped, or
 *     the like), 256-byte aligned, host_bytes >= GPUOS_STATIC_HOST_BYTES(queue_capacity).
 *     The library clears it.  It must stay untouched until gpuos_shutdown() has
 *     returned; gpuos_shutdown() does not free it.
 *   stream: a hipStream_t of the caller's on cfg.device (not the null stream; created
 *     non-blocking) that carries nothing but the worker until gpuos_shutdown(); the
 *     library does not destroy it.
 * All contexts made by this call on one GPU share that GPU's array, which keeps
 * what the previous one left: the call clears it, and only ONE such context can be
 * alive per GPU at a time: a second call before gpuos_shutdown() of the first
 * returns GPUOS_E_FULL instead of racing.  gpuos_worker_elapsed_ms is not available
 * on such a context (no events); every other call works as on any context
 * (gpuos_register_op and gpuos_define_program keep their audit records on the heap). */
#define GPUOS_STATIC_MAX_CAPACITY 1024
#define GPUOS_STATIC_HOST_BYTES(capacity) (65536ull + 512ull * (capacity))
int gpuos_init_static(gpuos_ctx** out, uint32_t queue_capacity, const gpuos_config* cfg,
                      void* host_block, uint64_t host_bytes, void* stream);

/* Operator table (paper Section 4.1 "Dynamic Operator Table"; dual-slot
 * update protocol).  Each logical op id owns two slots {impl, version} and a
 * version word; the active slot is version & 1.
 * register_op: first binding of op_id; fills the active slot, version = 1.
 * swap_op: writes {impl, version+1} into the INACTIVE slot, then publishes
 * version+1 with a store-release.  The worker never stops.  A task keeps the
 * slot and version it claimed; before a slot is overwritten the call waits
 * (bounded by wait_timeout_ms) until no unfinished task can still hold it.
 * The new impl must have the arity and kind (elementwise / reduction / row
 * operation) of the old one, or be GPUOS_IMPL_FAIL.  *out_version (nullable) gets the version.
 * Tasks submitted after the call returns observe a version >= *out_version. */
int gpuos_register_op(gpuos_ctx* ctx, uint32_t op_id, uint32_t impl_id, uint32_t* out_version);
int gpuos_swap_op(gpuos_ctx* ctx, uint32_t op_id, uint32_t impl_id, uint32_t* out_version);

/* Define an operator program (see enum gpuos_opcode): code: HOST array of
 * n_instr (1..32) instructions, copied; n_inputs: 1..3 tensor inputs the
 * operator takes.  *out_impl_id receives an implementation id that
 * gpuos_register_op and gpuos_swap_op accept (kind: elementwise, arity:
 * n_inputs).  A context holds at most GPUOS_MAX_PROGRAMS programs; they live
 * until shutdown (GPUOS_E_FULL when the table is full, GPUOS_E_INVAL for a
 * malformed program).  May be called while the worker runs and tasks are in
 * flight.  gpuos_launch_per_op, gpuos_task_plan and gpuos_task_bytes know
 * built-in implementations only. */
int gpuos_define_program(gpuos_ctx* ctx, const gpuos_instr* code, uint32_t n_instr, uint32_t n_inputs,
                         uint32_t* out_impl_id);

/* Paper Section 4.2: acquire n consecutive tickets, write the packed records
 * into their slots (slot = ticket & (capacity-1)).  tasks: HOST array of n
 * descriptors holding DEVICE tensor pointers.  All n are validated before
 * anything is written: on GPUOS_E_INVAL / GPUOS_E_BADOP nothing is enqueued.
 * The records become visible to the device at the next gpuos_flush (the
 * paper's fuse(): one aggregated submission).  When the ring is full the call
 * publishes what it has written and blocks until slots free up (or returns
 * GPUOS_E_FULL with nothing enqueued in non-blocking mode).  If that wait
 * ends in GPUOS_E_TIMEOUT or GPUOS_E_DEAD, the tasks written before it stay
 * enqueued and keep their tickets (gpuos_peek_queue's head_submitted minus
 * *out_first_ticket says how many); the rest were not submitted.
 * *out_first_ticket (nullable) receives the ticket of tasks[0]. */
int gpuos_submit(gpuos_ctx* ctx, const gpuos_task* tasks, uint32_t n, uint64_t* out_first_ticket);

/* Doorbell: one store-release of the tail cursor publishes every record
 * written so far.  Never waits for the device. */
int gpuos_flush(gpuos_ctx* ctx);

/* gpuos_submit followed by gpuos_flush (Section 4.2: write, then commit), as one call.  With the
 * ring in device memory a lone record (n = 1) and the doorbell then leave the caller's
 * write-combining buffers with one flush instead of two (0.1 us of a lone task's latency); the
 * doorbell may reach the device before the record, and the dispatcher reads a record that the
 * doorbell covers until its check word holds.  Same arguments, results and blocking behaviour as
 * gpuos_submit. */
int gpuos_submit_flush(gpuos_ctx* ctx, const gpuos_task* tasks, uint32_t n, uint64_t* out_first_ticket);

/* Flush, then block until `ticket` and every earlier ticket completed
 * (GPUOS_ALL: everything submitted).  timeout_ns == 0 uses wait_timeout_ms.
 * Returns the ticket's device status (for GPUOS_ALL: the first non-OK status
 * among tickets completed since the previous GPUOS_ALL wait), or
 * GPUOS_E_TIMEOUT / GPUOS_E_DEAD. */
int gpuos_wait(gpuos_ctx* ctx, uint64_t ticket, uint64_t timeout_ns);

/* Copy the completion records of tickets [first_ticket, first_ticket + n) to
 * the HOST array out.  Every ticket must be complete and still inside the
 * completion log, else GPUOS_E_INVAL. */
int gpuos_get_completions(gpuos_ctx* ctx, uint64_t first_ticket, uint32_t n, gpuos_completion* out);

/* Paper Table 1: peek_queue(), worker_alive() (1 alive, 0 not),
 * set_yield_every(every): every `every` polls with an empty ring the workers
 * sleep longer (0 = never yield: pure spin with short back-off). */
int gpuos_peek_queue(gpuos_ctx* ctx, gpuos_queue_state* out);
int gpuos_worker_alive(gpuos_ctx* ctx);
int gpuos_set_yield_every(gpuos_ctx* ctx, uint32_t every);

/* Paper Table 1 shutdown(): drain everything submitted, signal the worker to
 * exit, join the kernel, free the library's memory.  Idempotent on NULL. */
int gpuos_shutdown(gpuos_ctx* ctx);

/* Performance counters of the persistent kernel (paper Section 5.3), valid after
 * gpuos_stop_worker.  The counts are always kept; the times are zero unless
 * cfg.phase_timers was set.  out[0..15] (HOST array): dispatcher batches, records, work
 * units, then dispatcher time staging / resolving / writing / busy in 10 ns ticks,
 * dispatcher polls; then summed over all worker workgroups: work units executed
 * and 10 ns ticks spent waiting for work, fetching descriptors, waiting for
 * dependencies, executing, completing, and alive in total; out[15]: tasks the
 * dispatcher held back until their dependencies had completed. */
int gpuos_worker_stats(gpuos_ctx* ctx, uint64_t out[16]);

/* Milliseconds the worker kernel ran, from HIP events on its stream (valid
 * after the worker has exited, i.e. call it on a context being shut down via
 * gpuos_stop_worker).  gpuos_stop_worker drains and joins the kernel but keeps
 * the context so that timing and logs can still be read; gpuos_shutdown frees. */
int gpuos_stop_worker(gpuos_ctx* ctx);
int gpuos_worker_elapsed_ms(gpuos_ctx* ctx, float* out_ms);

/* Launch the worker again on a context whose worker has left: after
 * gpuos_stop_worker, or after it exited by itself (cfg.idle_exit_ms).  Tickets,
 * the completion log, the operator table (swaps made while it was stopped
 * included), programs and counters continue; gpuos_worker_elapsed_ms then covers
 * the latest run only.  This is how a caller hands the whole GPU to a kernel that
 * cannot start beside the worker (see the conventions at the top) and takes it
 * back: stop, run that kernel, start.  Tasks that were published just as the worker
 * left by itself (their gpuos_wait reports GPUOS_E_DEAD) are still in the ring and
 * are executed by the new run: start the worker, wait again.  GPUOS_OK also when the
 * worker is running; GPUOS_E_DEAD if the earlier run lost work or could not be joined.  Like
 * init / stop / shutdown: one thread, and no other thread inside a call. */
int gpuos_start_worker(gpuos_ctx* ctx);

/* Submit tasks[0..n) one at a time, waiting for each before the next is submitted, and
 * store each task's submit -> completion-seen host nanoseconds into lat_ns (HOST array of n,
 * nullable): the unloaded per-operation latency (paper Section 6.2), measured the same way as
 * the sync_each mode of gpuos_launch_per_op. */
int gpuos_run_serial(gpuos_ctx* ctx, const gpuos_task* tasks, uint32_t n, uint64_t* lat_ns);

/* The comparison the paper's evaluation is built on (Section 6: the same
 * operations issued as ordinary kernel launches): run the stream as ONE
 * hipLaunchKernel per task on one stream of `device`, with the library's own
 * operator code.  impl_of_op: HOST array of GPUOS_MAX_OPS impl ids (the table
 * contents to use).  sync_each = 0: one stream synchronize at the end;
 * 1: synchronize after every launch and store per-task launch->done host
 * nanoseconds into lat_ns (HOST array of n, nullable).  *out_seconds gets the
 * wall time of the whole stream. */
int gpuos_launch_per_op(int32_t device, const gpuos_task* tasks, uint32_t n,
                        const uint32_t* impl_of_op, int32_t sync_each,
                        uint64_t* lat_ns, double* out_seconds);

/* Measurement helper for the many-producers case (Section 6.4): n_threads host
 * threads started by the library submit tasks[0 .. n) to ctx at the same time,
 * thread k its contiguous share in batches of `batch` (one doorbell per
 * batch), `passes` times over (n_threads = 1: the calling thread does it, no
 * thread is started); the call returns when every thread has
 * submitted everything (it does not wait for completion: call gpuos_wait).
 * *out_seconds (nullable): wall time from the start of the threads to the
 * last submit returning.  Tasks must not depend on each other. */
int gpuos_submit_from_threads(gpuos_ctx* ctx, const gpuos_task* tasks, uint32_t n, uint32_t n_threads,
                              uint32_t batch, uint32_t passes, double* out_seconds);

/* Algorithmic HBM bytes of a task (tensor bytes the operation itself must
 * move: each distinct input element once, each output element once). */
int gpuos_task_bytes(const gpuos_task* task, uint32_t impl_id, uint64_t* out_bytes);

/* Observability (paper Section 5.3), available when cfg.trace_entries > 0,
 * else GPUOS_E_INVAL.
 * gpuos_get_trace: trace records of tickets [first_ticket, first_ticket + n),
 * which must be complete (wait for them first) and among the last
 * trace_entries tickets; out: HOST array of n.  GPUOS_E_INVAL if a record has
 * been overwritten by a later ticket or is not there yet.
 * gpuos_op_counts: tasks dispatched so far per operator id, as of the
 * dispatcher's last flush (it flushes whenever the ring runs empty and every
 * 256 batches); out: HOST array of GPUOS_MAX_OPS.
 * gpuos_trace_origin: host steady_clock nanoseconds (the clock of
 * gpuos_completion) at device tick 0, to within the latency of one device
 * write to host memory. */
int gpuos_get_trace(gpuos_ctx* ctx, uint64_t first_ticket, uint32_t n, gpuos_trace_record* out);
int gpuos_op_counts(gpuos_ctx* ctx, uint64_t* out);
int gpuos_trace_origin(gpuos_ctx* ctx, uint64_t* host_ns);

/* Kill switch (paper Section 5.3): rebind op_id to the stub that fails every
 * task at once with GPUOS_E_BADOP and writes nothing; the same as
 * gpuos_swap_op(ctx, op_id, GPUOS_IMPL_FAIL, out_version).  A later swap_op
 * to a real implementation brings the operator back. */
int gpuos_kill_op(gpuos_ctx* ctx, uint32_t op_id, uint32_t* out_version);

/* Audit log of the operator table (paper Section 4.4: every injection is
 * recorded for later review): one record per successful gpuos_register_op,
 * gpuos_swap_op, gpuos_kill_op and gpuos_define_program, in the order they took
 * effect.  head_ticket = tickets submitted before the change: every task from
 * that ticket on observes it (earlier ones may).  A program is recorded with
 * its length, arity and the FNV-1a hash (64 bit) of its instruction bytes.
 * The context keeps the latest 65,536 records.  out: HOST array of n records
 * starting at record number `first` (counted from the context's first change);
 * *out_total (may be NULL): records written so far.  GPUOS_E_INVAL if the range
 * is not (any longer) there. */
enum gpuos_audit_kind { GPUOS_AUDIT_REGISTER = 1, GPUOS_AUDIT_SWAP = 2, GPUOS_AUDIT_KILL = 3, GPUOS_AUDIT_DEFINE_PROGRAM = 4 };
typedef struct gpuos_audit_record {
  uint64_t t_ns;          /* host steady_clock nanoseconds (the clock of gpuos_completion) */
  uint64_t head_ticket;
  uint32_t kind;          /* enum gpuos_audit_kind                          */
  uint32_t op_id;         /* logical operator; 0 for DEFINE_PROGRAM         */
  uint32_t impl_id;       /* implementation bound, or the id the program got */
  uint32_t version;       /* the operator's version after the change; 0 for DEFINE_PROGRAM */
  uint32_t n_instr;       /* DEFINE_PROGRAM, and changes that bind a program */
  uint32_t n_inputs;
  uint64_t code_hash;
} gpuos_audit_record;     /* 48 bytes */
int gpuos_audit_log(gpuos_ctx* ctx, uint64_t first, uint32_t n, gpuos_audit_record* out, uint64_t* out_total);

/* How the host would hand this task to the workers (no GPU needed): out[0] =
 * execution path (0 nothing to do, 1 contiguous vector, 2 [rows, cols]
 * with row-vector / per-row-scalar operands, 3 generic strided walk,
 * 4 contiguous-row reduction, 5 generic reduction, 6 LDS-tiled transposed
 * gather, 7 row operation with rows in registers, 8 row operation over any
 * strides, 9 contiguous output with strided / broadcast / mixed-dtype inputs
 * gathered through LDS),
 * out[1] = work units (chunks) the task is split into, out[2] = size of one
 * unit in the path's own unit (elements, rows or 32 x 32 tiles), out[3] =
 * dims left after merging adjacent dims.  For tests and for sizing. */
int gpuos_task_plan(const gpuos_task* task, uint32_t impl_id, uint32_t out[4]);

/* Properties of `device` as the HIP runtime reports them (for reports; the
 * figures the roofline is priced against are the published ones, not these):
 * out[0] compute units, out[1] core clock kHz, out[2] memory clock kHz,
 * out[3] memory bus width bits, out[4] device memory bytes, out[5] L2 bytes,
 * out[6] LDS bytes per workgroup, out[7] wavefront size.  name: HOST buffer
 * of name_len bytes, always NUL-terminated (nullable). */
int gpuos_device_info(int32_t device, uint64_t out[8], char* name, uint32_t name_len);

const char* gpuos_strerror(int status);
const char* gpuos_last_hip_error(void);   /* text of the last failed HIP call     */

/* sizeof / offsetof facts of this ABI, for bindings to check their mirror of
 * the structs: out[0..7] = sizeof(gpuos_task), sizeof(gpuos_tensor),
 * offsetof(task,size), offsetof(task,in), offsetof(task,out),
 * offsetof(task,alpha), offsetof(task,dep), sizeof(gpuos_completion). */
void gpuos_abi_layout(uint32_t out[8]);

#ifdef __cplusplus
}
#endif
#endif /* GPUOS_H_ */
