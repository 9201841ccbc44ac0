// gpuos_internal.h -- layouts shared by the host runtime and the device code of
// the library: the packed 256-byte ring record, the control blocks and the
// operator-table entries.  Not part of the public ABI.
#pragma once
#if !defined(__HIPCC_RTC__)
#include <stdint.h>
#endif

#if defined(__HIP__)
#define GPUOS_HD __host__ __device__
#else
#define GPUOS_HD
#endif

namespace gpuos {

// How the executor walks a task (decided on the host after dim coalescing).
enum Path : uint8_t {
  PATH_NOP = 0,          // empty tensor: completes without touching memory
  PATH_CONTIG = 1,       // every operand contiguous 1-D, same dtype
  PATH_ROW2D = 2,        // [R, C] contiguous output; each input is full, a row vector
                         // broadcast over rows, or one scalar per row
  PATH_GENERIC = 3,      // index decomposition over <= 6 dims, any strides / dtypes
  PATH_RED_CONTIG = 4,   // last-dim reduction of a contiguous [rows, n] input
  PATH_RED_GENERIC = 5,  // last-dim reduction, any strides
  PATH_TILE2D = 6,       // [R, C] contiguous output, >= 1 input stored transposed:
                         // gathered through an LDS tile
  PATH_ROW_FUSED = 7,    // row operation (softmax, layer norm): contiguous rows of whole
                         // 16-byte vectors, one dtype, a row lives in one wavefront's registers
  PATH_ROW_GENERIC = 8,  // row operation over any strides / dtypes: three passes over memory
  PATH_STAGED = 9        // contiguous [R, C] output, inputs with any row / column strides (stride-2
                         // slices, row and column vectors, mixed dtypes): gathered through LDS
};

enum RecFlag : uint8_t {
  RF_FENCE = 1,          // dispatcher: publish only after every earlier ticket is done
  RF_VEC = 2,            // 16-byte vector access is safe (alignment and extents checked)
  RF_INT = 4,            // all tensors are I32
  RF_DEPS_RESOLVED = 8   // set by the dispatcher: published only after the dependencies completed
};

enum OperandKind : uint8_t { K_FULL = 0, K_ROWVEC = 1, K_ROWSCALAR = 2, K_TRANSPOSED = 3,
                             K_PERIODIC = 4 };   // PATH_ROW_FUSED: contiguous [period, n] block reused every `period` rows

constexpr uint32_t kMaxChunksPerTask = 1024;   // unit ring holds capacity * this entries
constexpr uint32_t kChunkElems = 16384;        // minimum elements per chunk
constexpr uint32_t kDispatchBatch = 64;        // records mirrored per dispatcher pass
constexpr uint32_t kThreads = 256;             // threads per workgroup of the worker

// The ring record ("compact descriptor", paper Section 4.1).  Written by the
// host into the host ring; the dispatcher copies it into the device mirror and
// fills impl / version / sel / status from the operator table.
struct alignas(16) Record {
  uint16_t op_id;
  uint8_t  path;
  uint8_t  ndim;             // after coalescing
  uint8_t  n_inputs;
  uint8_t  dtype[4];         // in0, in1, in2, out
  uint8_t  rflags;
  uint8_t  okind[3];         // PATH_ROW2D / PATH_TILE2D: OperandKind per input
  uint8_t  sel;              // table slot the task claimed            (dispatcher)
  uint16_t pad0;
  uint32_t impl;             // implementation id                     (dispatcher)
  uint32_t version;          // table version the task claimed        (dispatcher)
  int32_t  status;           // 0, or the error the task completes with (dispatcher)
  uint32_t nchunks;
  uint32_t chunk;            // elements (elementwise) or rows (reduction, row operation) per chunk
  uint32_t numel;            // elementwise: output elements; reduction / row operation: rows
  uint32_t red_n;            // reduction / row length
  float    alpha;
  uint16_t dep[3];
  uint16_t pad1;
  uint64_t ticket;
  uint64_t ptr[4];           // in0, in1, in2, out (device addresses)
  uint32_t size[6];          // coalesced iteration shape (reductions: outer dims)
  uint32_t stride[4][6];     // elements; 0 on broadcast dims; reductions and row operations:
                             // stride[k][5] is operand k's stride along the last dim, dims
                             // 0..ndim-1 are the outer dims; PATH_ROW_FUSED: stride[k][0] is
                             // the period (rows) of a K_PERIODIC input
  uint32_t t_dequeue[2];     // device clock when the dispatcher took the task (lo, hi)  (dispatcher)
  uint32_t pad2[7];
  uint32_t check;            // makes record_check_sum() of the record equal record_check_seed(ticket);
                             // set by the host, with the ticket field zero
};
static_assert(sizeof(Record) == 256, "ring record must be 256 bytes");

// Check word of a ring record.  With write-combined stores from several producer threads the
// pieces of a record reach device memory in any order, so the dispatcher may read any mixture
// of the record a slot held on the previous lap and the one being written.  The check is a
// weighted sum of the 64 words (word k times an odd constant of its own; the check word itself
// times 1) that must equal a seed derived from the ticket alone.  Position-dependent weights:
// two stale pointers that moved by the same amount do not cancel (they do under a plain xor).
// The ticket enters ONLY through the seed: the record's own ticket field is zero in the ring (the
// dispatcher fills it in); were it among the summed words, the previous lap's contents and check
// word would still verify under the new ticket word.
GPUOS_HD inline uint32_t record_check_weight(uint32_t k) { return k == 63u ? 1u : (2u * k + 1u) * 0x9E3779B1u; }
GPUOS_HD inline uint32_t record_check_seed(uint64_t ticket) {
  const uint64_t m = (ticket + 0x9E3779B97F4A7C15ull) * 0xD6E8FEB86659FD93ull;
  return (uint32_t)(m >> 32) ^ (uint32_t)m ^ 0x9E3779B9u;
}
// sum over words [0, n) of word * weight (n = 64: the value an intact record gives == its seed)
GPUOS_HD inline uint32_t record_check_sum(const uint32_t* words, uint32_t n) {
  uint32_t x = 0;
  for (uint32_t k = 0; k < n; ++k) x += words[k] * record_check_weight(k);
  return x;
}

// Completion word (8 bytes, one atomic store to host memory):
//   bits 0..31  low half of ticket+1, bits 32..39 status (int8), bits 40..63 version
GPUOS_HD inline uint64_t pack_completion(uint64_t ticket, int32_t status, uint32_t version) {
  return ((ticket + 1) & 0xffffffffull) | ((uint64_t)(uint8_t)(int8_t)status << 32) |
         ((uint64_t)(version & 0xffffffu) << 40);
}

// Operator-table entry: {impl, version} in one 64-bit word so that it can never tear.
GPUOS_HD inline uint64_t pack_entry(uint32_t impl, uint32_t version) { return ((uint64_t)version << 32) | impl; }

struct OpSlots {             // one logical operator: two slots + the version word
  uint64_t slot[2];          // active slot = version & 1
  uint32_t version;          // 0 = unregistered
  uint32_t pad;
};

// Control words.  HostCtl is written by the device and read by the host: it always lives in
// fine-grained host memory.  DoorbellCtl is written by the host and polled by the dispatcher: it
// lives in fine-grained host memory (the device polls over PCIe) or, in push mode, in device
// memory that the host writes through the PCIe BAR (the device polls its own HBM).
struct HostCtl {
  alignas(64) uint64_t dispatched;   // device -> host: tickets dequeued from the ring
  alignas(64) uint64_t heartbeat;    // device -> host: dispatcher poll counter
  alignas(64) uint32_t exit_code;    // device -> host: 0 running, 1 stop seen, 2 idle exit
  alignas(64) uint64_t clock_origin; // device -> host: the device clock when the dispatcher started
  alignas(64) uint32_t jit_alive;    // device -> host: generation of the run-time kernel whose workers are running
};
struct DoorbellCtl {
  // The dispatcher reads both words with ONE 16-byte load: the two are then sampled at the same
  // moment, and a tail value that covers a task submitted after a table change returned is never
  // seen together with the epoch from before that change (the host stores the epoch first).
  alignas(64) uint64_t tail;         // host -> device: tickets published (doorbell)
  uint64_t epoch_word;               // host -> device: epoch << 12 | op << 4 | stop bit;
                                     // op = 0xff: refresh every entry
  alignas(64) uint32_t yield_every;  // host -> device
  uint32_t jit_gen;                  // host -> device: generation of run-time kernel that is wanted (earlier ones leave)
};

struct DevCtl {                      // device memory
  alignas(128) uint64_t claim;       // next work unit to hand out (fetch-add)
  alignas(128) uint64_t tail_units;  // work units published by the dispatcher
  alignas(128) uint64_t done_count;  // tasks completed
  alignas(128) uint32_t stop_dev;    // dispatcher -> workers
  uint32_t yield_every;
  uint32_t jit_gen;                  // dispatcher -> workers of run-time kernels: the generation that is wanted (relayed from the doorbell block)
  alignas(128) uint64_t claim_j;     // second unit ring (tasks of natively compiled programs): next unit to hand out
  alignas(128) uint64_t tail_units_j;// ... units published on it (kept by the dispatcher, stored when it leaves)
  alignas(128) uint64_t jit_units;   // ... units executed from it so far
  // performance counters (paper Section 5.3), 100 MHz ticks; workers add theirs when they exit
  alignas(128) uint64_t stat[16];
};
enum StatIndex {
  ST_DISP_BATCHES = 0, ST_DISP_RECORDS, ST_DISP_UNITS, ST_DISP_TICKS_STAGE, ST_DISP_TICKS_RESOLVE,
  ST_DISP_TICKS_WRITE, ST_DISP_TICKS_TOTAL_BUSY, ST_DISP_POLLS,
  ST_WORK_UNITS = 8, ST_WORK_TICKS_WAIT, ST_WORK_TICKS_FETCH, ST_WORK_TICKS_DEP, ST_WORK_TICKS_EXEC,
  ST_WORK_TICKS_COMPLETE, ST_WORK_TICKS_TOTAL, ST_DISP_DEFERRED
};

struct SlotState {                   // device memory, one per ring slot
  uint64_t done_seq;                 // ticket+1 of the last task completed in this slot
  uint32_t chunks_done;
  uint32_t pad;
  uint64_t t_first;                  // tracing: device clock when chunk 0 of the current task was claimed
};

// One operator program as the device reads it (device-visible memory written by the host).
// The header is written after the code: ready == kProgramReady means the code is complete.
constexpr uint32_t kProgramReady = 0x50524f47u;
struct ProgramImage {
  uint32_t n_instr, n_inputs, ready;
  uint32_t native;            // 1: a run-time kernel that holds this program as native code is serving the second ring
  uint32_t code[2 * GPUOS_PROGRAM_MAX_INSTR];   // per instruction: op | dst << 8 | a << 16 | b << 24, then imm bits
};
static_assert(sizeof(ProgramImage) == 272, "program image layout");

struct TraceRec {                    // = gpuos_trace_record (48 bytes), host memory, one per traced ticket
  uint64_t ticket, t_dequeue, t_start, t_done;
  uint32_t op_version;
  uint16_t op_id;
  int8_t status;
  uint8_t reserved;
  uint32_t nchunks, workgroup;
};
static_assert(sizeof(TraceRec) == 48, "trace record layout");

// Work-unit entry: bits 0..9 chunk, 10..19 lap of the task's ticket around the ring (low 10 bits),
// 20..35 ring slot, 36..43 op id, 44 table slot, 45 op id valid, 46..63 stamp.  The stamp is the
// lap of the unit ring plus one (18 bits): the entry doubles as its own ready flag, so a worker that
// claimed unit g polls just that entry.  The ticket lap lets the worker tell the mirror record it is
// after from what the slot held a lap earlier (see mirror_record_valid).
GPUOS_HD inline uint64_t unit_stamp(uint64_t g, uint32_t unit_shift) { return ((g >> unit_shift) + 1) & 0x3ffffull; }
GPUOS_HD inline uint64_t pack_unit(uint32_t chunk, uint32_t lap, uint32_t slot, uint32_t op, uint32_t sel, uint32_t valid, uint64_t stamp) {
  return (uint64_t)(chunk & 0x3ffu) | ((uint64_t)(lap & 0x3ffu) << 10) | ((uint64_t)slot << 20) | ((uint64_t)(op & 0xff) << 36) |
         ((uint64_t)(sel & 1) << 44) | ((uint64_t)(valid & 1) << 45) | (stamp << 46);
}
static_assert(kMaxChunksPerTask <= 1024, "a chunk index has 10 bits in a work unit");

// The mirror of the ring is written by the dispatcher with sixteen 16-byte stores per record that
// land in any order, and the work units that name a record are published WITHOUT waiting for those
// stores (that wait was a memory round trip in every dispatcher pass and in every lone task's
// latency).  Instead the record proves itself: the dispatcher recomputes the check word over the
// record as it leaves (resolved fields and ticket included), and a worker accepts what it fetched
// only if the weighted sum equals the seed of the record's own ticket AND that ticket is the one the
// unit names (same slot, same lap); anything else (pieces of the record the slot held a lap ago) is
// fetched again.
GPUOS_HD inline bool mirror_record_valid(uint32_t sum, uint64_t ticket, uint32_t slot, uint32_t lap10, uint32_t cap_mask, uint32_t cap_shift) {
  return sum == record_check_seed(ticket) && (uint32_t)(ticket & cap_mask) == slot && (uint32_t)((ticket >> cap_shift) & 0x3ffu) == lap10;
}

struct WorkerArgs {
  HostCtl*   h;
  const DoorbellCtl* bell;
  const Record* hring;       // host ring (device-visible address)
  uint64_t*  hcomp;          // host completion words, one per slot
  const OpSlots* htable;     // host operator table
  DevCtl*    d;
  Record*    dring;          // device mirror of the ring
  uint64_t*  units;          // work-unit ring
  uint64_t*  units_j;        // second work-unit ring, same size (nullptr: no run-time kernels on this context)
  SlotState* st;
  OpSlots*   dtable;         // device-resident operator table
  uint32_t   cap_mask;
  uint32_t   unit_mask;
  uint32_t   unit_shift;     // log2 of the unit ring size
  uint32_t   cap_shift;      // log2 of the ring capacity
  uint64_t   idle_exit_ticks;   // 0 = never; 100 MHz ticks
  const ProgramImage* progs; // GPUOS_MAX_PROGRAMS images, written by the host
  TraceRec*  trace;          // host memory; nullptr = tracing off
  uint64_t*  opcount;        // host memory, GPUOS_MAX_OPS totals (tracing only)
  uint32_t   trace_mask;
  uint32_t   resume;         // 1: the context has run before; its counters continue where they stopped
  uint32_t   timing;         // 1: time every phase (performance counters); 0: read the clock only where tracing or the idle exit need it
  uint64_t   resume_tickets; // tickets dequeued (and completed) by the earlier runs
  uint64_t   dep_wait_ticks; // bound on a worker's wait for a dependency; 100 MHz ticks
};

// Where the device-side state of a context lies inside one block of device memory (the context
// created by gpuos_init_static keeps it in a file-scope device array instead of allocating it).
constexpr uint32_t kStaticMaxCapacity = 1024;
struct StaticLayout { size_t d, dring, units, st, dtable, total; };
constexpr size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
constexpr StaticLayout static_layout(uint32_t cap) {
  StaticLayout l{};
  l.d = 0;
  l.dring = align_up(l.d + sizeof(DevCtl), 256);
  l.units = align_up(l.dring + sizeof(Record) * cap, 256);
  l.st = align_up(l.units + sizeof(uint64_t) * (size_t)cap * kMaxChunksPerTask, 256);
  l.dtable = align_up(l.st + sizeof(SlotState) * cap, 256);
  l.total = align_up(l.dtable + sizeof(OpSlots) * GPUOS_MAX_OPS, 256);
  return l;
}
constexpr size_t kStaticScratchBytes = static_layout(kStaticMaxCapacity).total;   // about 8.3 MiB

// implemented in gpuos_kernels.hip
// Address, on `device`, of the file-scope device array that holds the device-side state of a
// context made by gpuos_init_static (each GPU has its own copy at its own address; looked up once
// per device).  Returns a hipError_t.
int static_scratch(int device, void** out);
int launch_worker(const WorkerArgs& a, uint32_t grid, void* stream);
// Before a worker is launched again on a context that has run before (same stream, ahead of it):
// the workgroups of the last run left with claims they never served.
int launch_resume_fixup(DevCtl* d, void* stream);
int worker_max_blocks_per_cu(int* out);
int launch_single(const Record& r, void* stream);   // one ordinary kernel launch for one task

}  // namespace gpuos
