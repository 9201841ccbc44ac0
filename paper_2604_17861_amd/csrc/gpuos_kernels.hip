// gpuos_kernels.hip -- device side of the GPUOS hot path for gfx950 (CDNA4).
//
//  * gpuos_worker_kernel: the persistent kernel (paper Section 4.1 "Persistent
//    Kernel Executor", device loop of Section 4.2).  Workgroup 0 is the
//    dispatcher: it is the single reader of the host ring (one PCIe poller
//    instead of hundreds), mirrors new records into device memory, resolves
//    each task's operator-table slot and version once ("claim time"), expands
//    tasks into work units (chunks) and publishes each with one 8-byte store
//    whose stamp makes it claimable (a lone new record takes the first
//    wavefront's short cut past the batch pass).  Every other workgroup is a
//    worker (run_worker in gpuos_device.h): its first wavefront claims work
//    units with an atomic fetch-add and holds up to eight descriptors, running
//    whichever is ready; the 4 wavefronts of the workgroup execute a chunk
//    together, and the last finisher of a task publishes its completion
//    (device-side done word for dependants, one 8-byte completion word to host
//    memory).
//  * gpuos_single_task_kernel: the same chunk executor as an ordinary kernel,
//    one launch per task (the per-op-launch comparison of the paper's Section 6).
//
// Wavefronts are 64 lanes; a workgroup is 256 threads.  Nothing here is a dense
// contraction, so there is no MFMA: the paths are bandwidth- or latency-bound
// and use 16-byte-per-lane global accesses, LDS for descriptor broadcast and
// cross-wave combines, and DPP / permute wave reductions.

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "../../include/gpuos.h"
#include "gpuos_internal.h"
#include "gpuos_device.h"

namespace gpuos {

// ---------------------------------------------------------------------------
// dispatcher (workgroup 0)
//
// Besides mirroring the host ring it is the scheduler of dependent work.  Units are claimed in
// publication order; a workgroup holds a few units at a time and runs whichever of them is ready, and
// when none is it can only wait.  Two rules keep that from hurting:
//  * A task with more than kSmallTaskChunks chunks whose dependencies are incomplete when it is
//    dequeued is HELD on a pending list and published when the done words say so (otherwise hundreds
//    of descriptor slots would be taken by it while ready work of other chains sits behind it).  Small
//    dependent tasks are published at once and wait, in the workgroups that claimed their units, on the
//    done word: the shortest hand-off for sequential chains of small operations.
//  * Publication order respects dependency order: a task that names a task which is itself not yet
//    published (it is on the pending list, or held earlier in the same pass) is held too, whatever its
//    size.  So whatever a waiting worker waits for lies BEFORE its own unit in the unit ring, its units
//    were claimed earlier by resident workgroups, and by induction over the ring position the wait
//    ends.  (Without this rule a held large task followed by more small dependants than the workgroups
//    can hold parks every workgroup behind units that come after theirs.)
// Held tasks are flagged RF_DEPS_RESOLVED: they are published only after their dependencies
// completed, so their workers never wait.
// ---------------------------------------------------------------------------
constexpr uint32_t kPendMax = 128;         // tasks held back at a time
constexpr uint64_t kLookaheadUnits = 8192; // work units kept published ahead of the claim counter
constexpr uint32_t kSmallTaskChunks = 4;
constexpr uint32_t kPrefetch = 4;          // records read together with every doorbell poll (4 x 16 lanes)
constexpr uint32_t kStageRetries = 4096;   // re-reads of a record that fails its check word (~ms) before it is failed

struct PubEntry {                          // what it takes to publish a task's work units
  uint32_t slot;
  uint32_t nchunks;
  uint32_t opinfo;                         // op id | table slot << 8 | valid << 9 | lap of the ticket (10 bits) << 16
  uint32_t route;                          // 0: main unit ring; 1: the second ring, served by the run-time kernel
};
struct PendEntry {
  uint64_t ticket;
  PubEntry pub;
  uint16_t dep[3];
  uint16_t pad;
};

// A staged record with a pitch of 68 words instead of 64: when the 64 lanes of a wavefront read the
// same field of 64 different records (the resolve and split steps do little else), a pitch of 64
// words puts all of them on one LDS bank; with 68 they spread over 16.
struct alignas(16) StagedRecord : Record {
  uint32_t pitch_pad[4];
};
static_assert(sizeof(StagedRecord) == 272, "staging pitch");

struct DispShared {
  StagedRecord rec[kDispatchBatch];        // 17 KB staging of the batch being mirrored
  uint64_t entry[GPUOS_MAX_OPS];           // shadow of the device table: current {impl, version}
  PubEntry pub[kDispatchBatch];            // tasks whose units are published in this pass (<= 64)
  uint32_t ubeg[kDispatchBatch + 1];       // exclusive prefix of their nchunks
  PendEntry pend[kPendMax];
  uint32_t defer[kDispatchBatch];          // per record of the batch: held back
  uint32_t bad[kDispatchBatch], ok[kDispatchBatch];   // staging: record still fails its check / passed on this read
  uint32_t nbad;
  uint32_t pre[kPrefetch];                 // prefetched with the poll and valid
  uint32_t preok[kDispatchBatch];          // requested while the previous batch was written out: arrived whole
  uint32_t opcnt[GPUOS_MAX_OPS];           // tracing: tasks dispatched per operator since the last flush
  uint32_t ready[kPendMax];                // per pending entry: dependencies complete
  uint32_t native[GPUOS_MAX_PROGRAMS];     // per operator program: 1 = its tasks go to the second ring (native code is being served there)
  uint64_t tail, epoch_word;
  uint32_t n, npend, npub, npub_second;
  uint64_t lane_tickets, lane_units;       // what the first wavefront's short cut for lone tasks has dispatched / published
  uint32_t lane_counted;                   // ... and whether it counted an operator (tracing)
};


DEV void dispatcher_refresh_native(const WorkerArgs& a, DispShared* s) {
  // which programs a run-time kernel serves natively, and which generation of it is wanted
  // (the host changes both only between two epoch bumps, and waits in between)
  const uint32_t tid = threadIdx.x;
  if (tid < GPUOS_MAX_PROGRAMS)
    s->native[tid] = (a.units_j != nullptr && a.progs != nullptr)
                         ? __hip_atomic_load(&a.progs[tid].native, __ATOMIC_RELAXED, SC_SYSTEM) : 0u;
  if (tid == GPUOS_MAX_PROGRAMS) {
    const uint32_t g = __hip_atomic_load(&a.bell->jit_gen, __ATOMIC_RELAXED, SC_SYSTEM);
    __hip_atomic_store(&a.d->jit_gen, g, __ATOMIC_RELAXED, SC_SYSTEM);
  }
}

DEV void dispatcher_refresh_table(const WorkerArgs& a, DispShared* s, uint32_t only_op) {
  // copy entries host table -> device table with the dual-slot protocol: the
  // inactive slot is written first, then the version is published.
  for (uint32_t op = threadIdx.x; op < GPUOS_MAX_OPS; op += kThreads) {
    if (only_op != 0xffu && op != only_op) continue;
    const uint32_t ver = __hip_atomic_load(&a.htable[op].version, __ATOMIC_RELAXED, SC_SYSTEM);
    if (ver == 0) continue;
    order_loads();
    const uint64_t e = __hip_atomic_load(&a.htable[op].slot[ver & 1u], __ATOMIC_RELAXED, SC_SYSTEM);
    if (e == s->entry[op]) continue;
    const uint32_t ev = (uint32_t)(e >> 32);
    __hip_atomic_store(&a.dtable[op].slot[ev & 1u], e, __ATOMIC_RELAXED, SC_SYSTEM);
    drain_stores();
    __hip_atomic_store(&a.dtable[op].version, ev, __ATOMIC_RELAXED, SC_SYSTEM);
    s->entry[op] = e;
  }
}

DEV bool deps_complete(const WorkerArgs& a, uint64_t ticket, const uint16_t* dep) {
  bool ok = true;
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    const uint32_t back = dep[k];
    if (back != 0 && back <= ticket) {
      const uint64_t want = ticket - back + 1;
      ok = ok && __hip_atomic_load(&a.st[(ticket - back) & a.cap_mask].done_seq, __ATOMIC_RELAXED, SC_SYSTEM) >= want;
    }
  }
  return ok;
}

// Does the task name a ticket that sits on the pending list (published later than everything the
// dispatcher has published so far)?  The list is in ticket order: two compares reject most
// candidates, a binary search decides the rest.
DEV bool names_pending(const DispShared* s, uint64_t ticket, const uint16_t* dep) {
  const uint32_t np = s->npend;
  if (np == 0) return false;
  const uint64_t first = s->pend[0].ticket, last = s->pend[np - 1].ticket;
  bool hit = false;
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    const uint32_t back = dep[k];
    if (back == 0 || back > ticket) continue;
    const uint64_t d = ticket - back;
    if (d < first || d > last) continue;
    uint32_t lo = 0, hi = np;
    while (lo < hi) {
      const uint32_t mid = (lo + hi) >> 1;
      if (s->pend[mid].ticket < d) lo = mid + 1; else hi = mid;
    }
    hit = hit || (lo < np && s->pend[lo].ticket == d);
  }
  return hit;
}

// Write the work units of s->pub[0 .. npub) and make them claimable.  Called by the whole
// workgroup; returns the number of units published.
// Ring `route` only: entries of the other ring count as zero units (they keep their place in the
// list, so both rings see their tasks in list order).
DEV uint32_t dispatcher_publish(const WorkerArgs& a, DispShared* s, uint32_t npub, uint64_t units_w, uint32_t route = 0) {
  const uint32_t tid = threadIdx.x;
  uint64_t* const ring = route == 0 ? a.units : a.units_j;
  if (tid < 64) {                                  // wave 0: inclusive scan of nchunks
    // inclusive scan over the wavefront with DPP: shifts by 1, 2, 4, 8 inside each row of 16 lanes
    // (lanes the shift runs out of the row for add 0), then lane 15 of a row to the whole next row
    // (rows 1 and 3), then lane 31 to rows 2 and 3.  Six shuffles through the LDS crossbar before.
    int v = (int)((tid < npub && s->pub[tid].route == route) ? s->pub[tid].nchunks : 0u);
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);
    s->ubeg[tid + 1] = (uint32_t)v;                // (entries past npub hold the total: the search below counts them out)
    if (tid == 0) s->ubeg[0] = 0;
  }
  __syncthreads();
  const uint32_t total = s->ubeg[npub];
  // (no wait for the mirror stores of this pass: a worker checks the record it fetches, see mirror_record_valid)
  for (uint32_t u = tid; u < total; u += kThreads) {
    // The task of unit u is the number of prefix entries 1..64 that are <= u (they only grow).  Counted
    // in two levels of seven independent reads each, two LDS latencies, where a binary search takes six.
    static_assert(kDispatchBatch == 64, "two levels of eight");
    uint32_t oct = 0;
#pragma unroll
    for (uint32_t k = 1; k < 8; ++k) oct += s->ubeg[8u * k] <= u ? 1u : 0u;
    uint32_t lo = 8u * oct;
#pragma unroll
    for (uint32_t j = 1; j < 8; ++j) lo += s->ubeg[8u * oct + j] <= u ? 1u : 0u;
    const PubEntry pe = s->pub[lo];
    const uint64_t g = units_w + u;
    // one 8-byte store publishes the unit: the stamp makes it claimable
    __hip_atomic_store(&ring[g & a.unit_mask],
                       pack_unit(u - s->ubeg[lo], pe.opinfo >> 16, pe.slot, pe.opinfo & 0xffu, (pe.opinfo >> 8) & 1u, (pe.opinfo >> 9) & 1u,
                                 unit_stamp(g, a.unit_shift)),
                       __ATOMIC_RELAXED, SC_SYSTEM);
  }
  __syncthreads();                                 // s->pub / s->ubeg may be rewritten after this
  return total;
}

struct UnitCursors { uint64_t w[2]; };      // units published so far on the main ring and on the second ring

// Publish s->pub[0 .. npub) on the ring(s) its entries name.  Called by the whole workgroup.
DEV void dispatcher_publish_all(const WorkerArgs& a, DispShared* s, uint32_t npub, UnitCursors& uc, bool any_second) {
  uc.w[0] += dispatcher_publish(a, s, npub, uc.w[0], 0);
  if (any_second) uc.w[1] += dispatcher_publish(a, s, npub, uc.w[1], 1);
}

// Publish the pending tasks whose dependencies have completed.
DEV void dispatcher_service_pending(const WorkerArgs& a, DispShared* s, UnitCursors& uc) {
  const uint32_t tid = threadIdx.x;
  const uint32_t np = s->npend;
  if (np == 0) return;
  static_assert(kPendMax <= 128 && kPendMax <= kThreads, "one pending entry per thread of the first two wavefronts");
  // One entry per thread: is it ready, and where does it go?  The first kDispatchBatch ready entries
  // move to the publish list, everything else closes ranks in the pending list; both keep their order
  // (ticket order).  Positions come from a ballot inside each of the two wavefronts plus the count
  // of the first one.
  const uint32_t lane = tid & 63u, wave = tid >> 6;
  PendEntry e;
  bool ready = false;
  if (tid < np) {
    e = s->pend[tid];
    ready = deps_complete(a, e.ticket, e.dep);
  }
  uint64_t m_ready = 0;
  if (tid < 128u) {
    m_ready = __ballot(ready);
    const uint64_t m_second = __ballot(ready && e.pub.route != 0);
    if (lane == 0) { s->ready[wave] = (uint32_t)__popcll(m_ready); s->ready[2 + wave] = m_second != 0 ? 1u : 0u; }
  }
  __syncthreads();                                 // the counts; and every entry is in its thread's registers
  const uint32_t ready0 = s->ready[0], ready_all = ready0 + s->ready[1];
  const bool any_second = (s->ready[2] | s->ready[3]) != 0;
  if (tid < np) {
    const uint32_t ready_before = (uint32_t)__popcll(m_ready & ((1ull << lane) - 1ull)) + (wave ? ready0 : 0u);
    const uint32_t taken_before = ready_before < kDispatchBatch ? ready_before : kDispatchBatch;
    if (ready && ready_before < kDispatchBatch) s->pub[ready_before] = e.pub;      // the rest waits for the next call
    else s->pend[tid - taken_before] = e;
  }
  const uint32_t npub = ready_all < kDispatchBatch ? ready_all : kDispatchBatch;
  __syncthreads();                                 // the lists are complete (and s->ready may be reused)
  if (tid == 0) s->npend = np - npub;
  if (npub == 0) { __syncthreads(); return; }
  order_loads();
  dispatcher_publish_all(a, s, npub, uc, any_second);   // its barriers also cover the new pending count
}

DEV void run_dispatcher(const WorkerArgs& a, DispShared* s) {
  const uint32_t tid = threadIdx.x;
  // A context whose worker was stopped and started again continues its ticket and work-unit
  // counts (both are zero on a fresh context); the operator table is read again from the host's
  // copy because the epoch seen starts at zero.
  uint64_t mirrored = a.resume_tickets, seen_epoch = 0;
  UnitCursors uc;
  uc.w[0] = __hip_atomic_load(&a.d->tail_units, __ATOMIC_RELAXED, SC_SYSTEM);
  uc.w[1] = __hip_atomic_load(&a.d->tail_units_j, __ATOMIC_RELAXED, SC_SYSTEM);
  for (uint32_t op = tid; op < GPUOS_MAX_OPS; op += kThreads) { s->entry[op] = 0; s->opcnt[op] = 0; }
  if (tid == 0) { s->npend = 0; s->lane_counted = 0; }
  __syncthreads();
  uint64_t idle_since = wall_clock64();
  if (tid == 0) {
    if (!a.resume) __hip_atomic_store(&a.h->clock_origin, idle_since, __ATOMIC_RELAXED, SC_SYSTEM);
    // the first heartbeat leaves together with the clock origin: the host pairs the moment it sees
    // it with device tick `clock_origin` (later heartbeats are poll counts, all above 1)
    __hip_atomic_store(&a.h->heartbeat, 1ull, __ATOMIC_RELAXED, SC_SYSTEM);
  }
  const bool tracing = a.trace != nullptr;
  const bool timing = a.timing != 0;
  uint32_t passes_since_flush = 0;
  bool counts_dirty = false;
  uint64_t polls = 0;
  bool stopping = false;
  uint64_t st_batches = 0, st_records = 0, st_units = 0, st_stage = 0, st_resolve = 0, st_write = 0, st_busy = 0;
  uint64_t st_deferred = 0;
  uint64_t claimed = uc.w[0];              // last value read from the claim counter (thread 0)
  constexpr uint32_t kStagePieces = kDispatchBatch * 16u / kThreads;      // 16-byte pieces of a batch per thread
  static_assert(kStagePieces * kThreads == kDispatchBatch * 16u, "a batch is staged in whole rounds of the workgroup");
  uint64_t pre_base = ~0ull;               // first ticket of the records requested ahead (they wait in s->rec)
  uint32_t pre_n = 0;                      // how many
  const rsrc_t rh = make_rsrc(a.hring, (a.cap_mask + 1u) * (uint32_t)sizeof(Record));
  const rsrc_t rd = make_rsrc(a.dring, (a.cap_mask + 1u) * (uint32_t)sizeof(Record));
  const rsrc_t rbell = make_rsrc(a.bell, 16u);
  static_assert(offsetof(DoorbellCtl, tail) == 0 && offsetof(DoorbellCtl, epoch_word) == 8, "tail and epoch word are read with one 16-byte load");
  while (true) {
    // ---- poll the host ring (wavefront 0; the only PCIe poller of the kernel) ----
    // Every poll also reads the next kPrefetch records of the ring in the same round trip.  When
    // the doorbell then shows them published and their check words hold, they are already staged:
    // a lone task reaches the workers after one PCIe read latency instead of two.
    if (tid < 64) {
      uint64_t t, e;
      v4i q;
      const uint32_t g = tid >> 4, part = tid & 15u;               // record g of the prefetch window, 16-byte piece
      const bool have_pending = s->npend != 0;
      bool lane_dirty = false;                         // the short cut below counted an operator (tracing) since the last flush
      struct Poll { uint64_t t, e; v4i q; };
      auto request = [&](uint64_t base) {
        Poll p;
        const uint32_t slot = (uint32_t)((base + g) & a.cap_mask);
        const v4i b = Mem<POL_COHERENT>::ld16(rbell, 0u);        // tail and epoch word, one sample of both
        p.t = ((uint64_t)(uint32_t)b[1] << 32) | (uint32_t)b[0];
        p.e = ((uint64_t)(uint32_t)b[3] << 32) | (uint32_t)b[2];
        p.q = Mem<POL_COHERENT>::ld16(rh, slot * (uint32_t)sizeof(Record) + part * 16u);
        return p;
      };
      while (true) {
        const Poll cur = request(mirrored);
        t = cur.t; e = cur.e; q = cur.q;
        ++polls;
        if (tid == 0 && (polls & 63u) == 0) __hip_atomic_store(&a.h->heartbeat, polls, __ATOMIC_RELAXED, SC_SYSTEM);
        if (t == mirrored + 1 && e == seen_epoch && !stopping && !have_pending) {
          // ---- short cut for a lone task ----
          // One new record, whole (its check word holds), no table change, nothing held back: this
          // wavefront resolves, mirrors and publishes it by itself and polls on.  The other three
          // stay at the barrier below; the dozen barriers of a batch pass are not on a lone task's
          // way.  Anything special (a dependency, a fence, many chunks, the second ring, a full
          // lookahead window) takes the ordinary way.
          order_loads();
          const uint32_t x0 = record_piece_sum(q, part);
          const uint32_t claimed_lo = __builtin_amdgcn_readfirstlane((uint32_t)claimed);
          const uint32_t claimed_hi = __builtin_amdgcn_readfirstlane((uint32_t)(claimed >> 32));
          const uint64_t claimed0 = ((uint64_t)claimed_hi << 32) | claimed_lo;       // thread 0 keeps the count
          bool lone = __builtin_amdgcn_readfirstlane((uint32_t)(x0 == record_check_seed(mirrored))) != 0 &&
                      !(uc.w[0] > claimed0 && uc.w[0] - claimed0 >= kLookaheadUnits);
          if (lone) {
            if (tid < 16) ((v4i*)&s->rec[0])[part] = q;
            lds_wave_sync();
            Record& rc = s->rec[0];
            const uint32_t op = uni(rc.op_id);
            uint32_t nch = uni(rc.nchunks);
            const uint64_t ent = op < GPUOS_MAX_OPS ? s->entry[op] : 0ull;
            const uint32_t impl = uni((uint32_t)ent);
            lone = (rc.rflags & RF_FENCE) == 0 && (rc.dep[0] | rc.dep[1] | rc.dep[2]) == 0 && nch <= 64u &&
                   impl < GPUOS_IMPL_PROGRAM_BASE;
            if (lone) {
              const int32_t status = ent == 0 ? GPUOS_E_BADOP : GPUOS_OK;        // (covers an op id out of range)
              if (status != GPUOS_OK || nch == 0) nch = 1;
              const uint32_t sel = (uint32_t)((ent >> 32) & 1u);
              const uint64_t tk0 = clock_if(tracing);
              lds_wave_sync();                                             // every lane has read what lane 0 overwrites
              if (tid == 0) {
                rc.impl = impl;
                rc.version = (uint32_t)(ent >> 32);
                rc.sel = (uint8_t)sel;
                rc.status = status;
                rc.nchunks = nch;
                rc.ticket = mirrored;
                if (tracing) {
                  rc.t_dequeue[0] = (uint32_t)tk0; rc.t_dequeue[1] = (uint32_t)(tk0 >> 32);
                  if (op < GPUOS_MAX_OPS) { atomicAdd(&s->opcnt[op], 1u); s->lane_counted = 1u; }
                }
              }
              lane_dirty = tracing;
              lds_wave_sync();
              const uint32_t slot0 = (uint32_t)(mirrored & a.cap_mask);
              if (tid < 16) {
                v4i w = ((const v4i*)&s->rec[0])[part];
                if (part == 15u) w[3] = 0;
                const uint32_t xs = record_piece_sum(w, part);
                if (part == 15u) w[3] = (int)(record_check_seed(mirrored) - xs);
                Mem<POL_COHERENT>::st16(rd, slot0 * (uint32_t)sizeof(Record) + part * 16u, w);
              }
              if (tid < nch) {
                const uint64_t gu = uc.w[0] + tid;
                __hip_atomic_store(&a.units[gu & a.unit_mask],
                                   pack_unit(tid, (uint32_t)((mirrored >> a.cap_shift) & 0x3ffu), slot0, op, sel, status == GPUOS_OK ? 1u : 0u,
                                             unit_stamp(gu, a.unit_shift)),
                                   __ATOMIC_RELAXED, SC_SYSTEM);
              }
              mirrored += 1;
              uc.w[0] += nch;
              if (tid == 0) __hip_atomic_store(&a.h->dispatched, mirrored, __ATOMIC_RELAXED, SC_SYSTEM);
              if (timing || a.idle_exit_ticks != 0) idle_since = wall_clock64();
              st_batches += 1; st_records += 1; st_units += nch;
              continue;
            }
          }
        }
        if (t != mirrored || e != seen_epoch || stopping || have_pending) break;
        if (lane_dirty && (polls & 63u) == 0) break;    // idle again: let the whole workgroup publish the per-operator counts
        if ((polls & 63u) == 0 && a.idle_exit_ticks != 0 && wall_clock64() - idle_since > a.idle_exit_ticks) {
          e |= 2u;                                  // behave as if the host had asked to stop
          break;
        }
      }
      order_loads();
      // keep the prefetched records whose check word holds and that the doorbell value read in the
      // same round covers
      const uint32_t x = record_piece_sum(q, part);
      const bool good = mirrored + g < t && x == record_check_seed(mirrored + g);
      if (good) ((v4i*)&s->rec[g])[part] = q;
      if (part == 0) s->pre[g] = good ? 1u : 0u;
      if (e & 3u) {                                 // stop: take the final tail after the flag
        t = __hip_atomic_load(&a.bell->tail, __ATOMIC_RELAXED, SC_SYSTEM);
        order_loads();
      }
      if (tid == 0) {
        s->tail = t;
        s->epoch_word = e;
        s->lane_tickets = mirrored;
        s->lane_units = uc.w[0];
      }
    }
    __syncthreads();
    const uint64_t tail = s->tail, ew = s->epoch_word;
    mirrored = s->lane_tickets;                      // the short cut above may have moved both on
    uc.w[0] = s->lane_units;
    if (tracing && s->lane_counted) counts_dirty = true;
    __syncthreads();
    if (tracing && tid == 0) s->lane_counted = 0;  // (read again only after the next poll's barrier)
    if ((ew >> 12) != (seen_epoch >> 12)) {
      const uint32_t hinted = (uint32_t)((ew >> 4) & 0xffu);
      const bool one = ((ew >> 12) - (seen_epoch >> 12)) == 1 && hinted != 0xffu;
      dispatcher_refresh_table(a, s, one ? hinted : 0xffu);
      dispatcher_refresh_native(a, s);
      if (tid == 0) {
        const uint32_t y = __hip_atomic_load(&a.bell->yield_every, __ATOMIC_RELAXED, SC_SYSTEM);
        __hip_atomic_store(&a.d->yield_every, y, __ATOMIC_RELAXED, SC_SYSTEM);
      }
      __syncthreads();
    }
    seen_epoch = ew & ~3ull;
    if (ew & 3u) stopping = true;

    dispatcher_service_pending(a, s, uc);

    // ---- mirror new records, batch by batch ----
    bool first_batch = true;                       // the prefetched records belong to the first batch after a poll
    while (mirrored < tail) {
      // Dequeue only a bounded distance ahead of execution: the dependency state seen at dequeue
      // time is then close to what the workers will see, and the pending list stays short.
      if (tid == 0) {
        // the claim counter only grows: re-read it only when the cached value says "too far ahead"
        if (uc.w[0] > claimed && uc.w[0] - claimed >= kLookaheadUnits)
          claimed = __hip_atomic_load(&a.d->claim, __ATOMIC_RELAXED, SC_SYSTEM);
        const uint32_t room = kPendMax - s->npend;
        uint32_t take = (uint32_t)((tail - mirrored) < kDispatchBatch ? (tail - mirrored) : kDispatchBatch);
        if (take > room) take = room;
        if (uc.w[0] > claimed && uc.w[0] - claimed >= kLookaheadUnits) take = 0;
        s->n = take;
      }
      __syncthreads();
      uint32_t n = s->n;                           // (written again only behind the barriers of staging, or of the next poll)
      if (n == 0) {                                                // throttled: let the workers catch up
        dispatcher_service_pending(a, s, uc);
        if (s->npend == 0) __builtin_amdgcn_s_sleep(8);
        break;                                                     // back to the poll loop (stop, table, heartbeat)
      }
      const uint64_t tk0 = clock_if(timing || tracing);
      // stage: 16 pieces of 16 bytes per record.  System-scope loads: an ordinary load of host
      // memory may hit a line the CU's vector cache kept from the previous lap of the ring.
      // Every record carries a check word (a weighted sum of its 64 words must equal a seed made
      // from its ticket): a record that has not landed completely yet, or is left over from the previous lap,
      // fails the check and is read again; one that never passes is completed with an error
      // instead of being executed.
      // Records requested ahead (with the poll, or while the previous batch was written out) already
      // lie in s->rec and were checked as they arrived: a batch made of such records only is staged
      // by one ballot and one barrier.  Everything else is read here, and read again until it checks.
      static_assert(kDispatchBatch == 64, "one wavefront looks at the whole batch");
      if (tid < kDispatchBatch) {
        const bool ahead = (pre_base == mirrored && tid < pre_n && s->preok[tid] != 0) || (first_batch && tid < kPrefetch && s->pre[tid] != 0);
        const bool bad = tid < n && !ahead;
        s->bad[tid] = bad ? 1u : 0u;
        const uint64_t m = __ballot(bad);
        if (tid == 0) s->nbad = (uint32_t)__popcll(m);
      }
      first_batch = false;
      __syncthreads();
      for (uint32_t attempt = 0; s->nbad != 0 && attempt < kStageRetries; ++attempt) {
#pragma unroll
        for (uint32_t j = 0; j < kStagePieces; ++j) {
          const uint32_t p = tid + j * kThreads;
          if (p < n * 16u) {
            const uint32_t rix = p >> 4, part = p & 15u;
            if (s->bad[rix]) {                                     // uniform over the 16 lanes of a record
              const uint32_t slot = (uint32_t)((mirrored + rix) & a.cap_mask);
              const v4i q = Mem<POL_COHERENT>::ld16(rh, slot * (uint32_t)sizeof(Record) + part * 16u);
              ((v4i*)&s->rec[rix])[part] = q;
              const uint32_t x = record_piece_sum(q, part);
              if (part == 0) s->ok[rix] = (x == record_check_seed(mirrored + rix)) ? 1u : 0u;
            }
          }
        }
        __syncthreads();
        if (tid < 64) {
          const bool still_bad = tid < n && s->bad[tid] && !s->ok[tid];
          if (tid < n && s->bad[tid] && s->ok[tid]) s->bad[tid] = 0;
          const uint64_t m = __ballot(still_bad);
          if (tid == 0) s->nbad = (uint32_t)__popcll(m);
        }
        __syncthreads();
        if (s->nbad == 0) break;
        __builtin_amdgcn_s_sleep(16);
      }
      const uint64_t tk1 = clock_if(timing);
      // a FENCE task starts a batch of its own: cut the batch in front of the first one after slot 0
      if (tid < 64) {
        const bool f = tid >= 1 && tid < n && (s->rec[tid].rflags & RF_FENCE);
        const uint64_t m = __ballot(f);
        if (tid == 0) s->n = m ? (uint32_t)__builtin_ctzll(m) : n;
      }
      __syncthreads();
      n = s->n;
      // Request the next batch now, if the doorbell value already covers it: the loads travel while
      // this batch is resolved, written to the mirror and published (2.5 us; behind the mirror and
      // publish steps alone the copy at the end of the pass still waited for them).  A piece that turns
      // out incomplete fails its record's check word when it arrives and is read again at staging time.
      pre_base = mirrored + n;
      pre_n = tail > pre_base ? (uint32_t)((tail - pre_base) < kDispatchBatch ? (tail - pre_base) : kDispatchBatch) : 0u;
      v4i pre_q[kStagePieces];
#pragma unroll
      for (uint32_t j = 0; j < kStagePieces; ++j) {
        // No branch round the load: a piece that is not wanted gets an offset past the ring, which the
        // buffer hardware answers with zero without touching memory.  (With the load under an `if`
        // the compiler waited for each of the four before it issued the next: four memory round
        // trips in a row, 1.6 of the pass's 4.4 us.)
        const uint32_t p = tid + j * kThreads;
        const uint32_t slot = (uint32_t)((pre_base + (p >> 4)) & a.cap_mask);
        pre_q[j] = Mem<POL_COHERENT>::ld16(rh, p < pre_n * 16u ? slot * (uint32_t)sizeof(Record) + (p & 15u) * 16u : kNoLoad);
      }
      // resolve the operator table ("claim time": slot, version, impl, status) and the dependencies
      if (tid < n) {
        Record& rc = s->rec[tid];
        const uint32_t op = rc.op_id;
        const uint64_t ticket = mirrored + tid;
        int32_t status = GPUOS_OK;
        uint64_t e = 0;
        if (s->bad[tid]) {                                         // never passed its check: do not trust any field
          status = GPUOS_E_INVAL;
          rc.path = PATH_NOP; rc.nchunks = 1; rc.dep[0] = rc.dep[1] = rc.dep[2] = 0; rc.rflags = 0;
        } else if (op >= GPUOS_MAX_OPS) status = GPUOS_E_BADOP;   // bounds check on the op id
        else {
          e = s->entry[op];
          if (e == 0) status = GPUOS_E_BADOP;                      // never registered
        }
        rc.impl = (uint32_t)e;
        rc.version = (uint32_t)(e >> 32);
        rc.sel = (uint8_t)((e >> 32) & 1u);
        rc.status = status;
        if (status != GPUOS_OK || rc.nchunks == 0) rc.nchunks = 1; // one unit reports the task
        rc.ticket = ticket;
        if (tracing) {
          rc.t_dequeue[0] = (uint32_t)tk0; rc.t_dequeue[1] = (uint32_t)(tk0 >> 32);
          if (op < GPUOS_MAX_OPS) atomicAdd(&s->opcnt[op], 1u);
        }
        uint32_t defer = 0;
        if ((rc.dep[0] | rc.dep[1] | rc.dep[2]) != 0) {
          if (rc.nchunks > kSmallTaskChunks) {
            // a large dependent task: its workers never wait; it is published once its
            // dependencies are complete (now, or later from the pending list)
            rc.rflags |= RF_DEPS_RESOLVED;
            defer = deps_complete(a, ticket, rc.dep) ? 0u : 1u;
          } else {
            // a small one is published at once and its workers wait, unless it names a task that is
            // itself held back: then it joins the pending list behind that task (tasks held in this
            // very pass are found below, in the split)
            defer = names_pending(s, ticket, rc.dep) ? 1u : 0u;
          }
        }
        s->defer[tid] = defer;
      }
      __syncthreads();
      // a leading FENCE: everything earlier must be published and complete first
      if (s->rec[0].rflags & RF_FENCE) {
        while (s->npend != 0) dispatcher_service_pending(a, s, uc);
        if (tid == 0) {
          while (__hip_atomic_load(&a.d->done_count, __ATOMIC_RELAXED, SC_SYSTEM) < mirrored)
            __builtin_amdgcn_s_sleep(4);
          order_loads();
        }
        __syncthreads();
      }
      if (tid < 64) {                                              // wave 0 holds all n <= 64 records: split by ballot
        const uint32_t npend0 = s->npend;
        const bool mine = tid < n;
        bool held = mine && s->defer[tid] != 0;
        // A task that names a task held in this pass is held too (a large one already is: such a
        // dependency cannot be complete).  Dependencies point backwards, so a few rounds of
        // "held if one of my in-pass dependencies is held" reach the fixed point.
        uint64_t dep_mask = 0;                                     // records of this pass the task names
        if (mine && !held) {
#pragma unroll
          for (int k = 0; k < 3; ++k) {
            const uint32_t back = s->rec[tid].dep[k];
            if (back != 0 && back <= tid) dep_mask |= 1ull << (tid - back);
          }
        }
        uint64_t m_def = __ballot(held);
        while (true) {
          held = held || (dep_mask & m_def) != 0;
          const uint64_t m2 = __ballot(held);
          if (m2 == m_def) break;
          m_def = m2;
        }
        const uint64_t m_pub = __ballot(mine && !held);
        const uint64_t below = (1ull << tid) - 1ull;
        bool second = false;                                       // published now, on the second ring
        if (held) s->rec[tid].rflags |= RF_DEPS_RESOLVED;          // published only after its dependencies completed
        if (mine) {
          const Record& rc = s->rec[tid];
          PubEntry pe;
          pe.slot = (uint32_t)((mirrored + tid) & a.cap_mask);
          pe.nchunks = rc.nchunks;
          pe.opinfo = (rc.op_id & 0xffu) | ((uint32_t)rc.sel << 8) | ((rc.status == GPUOS_OK ? 1u : 0u) << 9) |
                      ((uint32_t)(((mirrored + tid) >> a.cap_shift) & 0x3ffu) << 16);
          // tasks of a program that a run-time kernel holds as native code go to that kernel's ring
          const uint32_t prog = rc.impl - GPUOS_IMPL_PROGRAM_BASE;
          pe.route = (rc.status == GPUOS_OK && rc.impl >= GPUOS_IMPL_PROGRAM_BASE && prog < GPUOS_MAX_PROGRAMS && s->native[prog] != 0) ? 1u : 0u;
          second = pe.route != 0 && !held;
          if (held) {
            PendEntry& pd = s->pend[npend0 + (uint32_t)__popcll(m_def & below)];
            pd.ticket = mirrored + tid;
            pd.pub = pe;
            pd.dep[0] = rc.dep[0]; pd.dep[1] = rc.dep[1]; pd.dep[2] = rc.dep[2];
          } else {
            s->pub[(uint32_t)__popcll(m_pub & below)] = pe;
          }
        }
        const uint64_t m_second = __ballot(second);
        if (tid == 0) {
          st_deferred += (uint32_t)__popcll(m_def);
          s->npend = npend0 + (uint32_t)__popcll(m_def);
          s->npub = (uint32_t)__popcll(m_pub);
          s->npub_second = m_second != 0 ? 1u : 0u;
        }
      }
      __syncthreads();
      const uint64_t tk2 = clock_if(timing);
      // write the records into the device mirror (write-through stores), held-back ones included
      // each record leaves with a check word of its own over what it now holds (resolved fields, ticket)
      for (uint32_t p = tid; p < n * 16u; p += kThreads) {
        const uint32_t rix = p >> 4, part = p & 15u;
        const uint32_t slot = (uint32_t)((mirrored + rix) & a.cap_mask);
        v4i q = ((const v4i*)&s->rec[rix])[part];
        if (part == 15u) q[3] = 0;
        const uint32_t x = record_piece_sum(q, part);              // the 16 lanes of a record share a row
        if (part == 15u) q[3] = (int)(record_check_seed(mirrored + rix) - x);
        Mem<POL_COHERENT>::st16(rd, slot * (uint32_t)sizeof(Record) + part * 16u, q);
      }
      const uint64_t before = uc.w[0] + uc.w[1];
      dispatcher_publish_all(a, s, s->npub, uc, s->npub_second != 0);       // (no wait for the stores above: see mirror_record_valid)
      const uint32_t total = (uint32_t)(uc.w[0] + uc.w[1] - before);
      // nothing reads this batch's staging any more (the mirror has it, held-back tasks were copied
      // to the pending list): it takes the records requested ahead
      // (and each is checked as it arrives: the next pass finds the verdict in s->preok)
#pragma unroll
      for (uint32_t j = 0; j < kStagePieces; ++j) {
        const uint32_t p = tid + j * kThreads;
        if (p < pre_n * 16u) {                                       // uniform over the 16 lanes of a record
          ((v4i*)&s->rec[p >> 4])[p & 15u] = pre_q[j];
          const uint32_t x = record_piece_sum(pre_q[j], p & 15u);
          if ((p & 15u) == 0) s->preok[p >> 4] = (x == record_check_seed(pre_base + (p >> 4))) ? 1u : 0u;
        }
      }
      mirrored += n;
      if (tid == 0) __hip_atomic_store(&a.h->dispatched, mirrored, __ATOMIC_RELAXED, SC_SYSTEM);
      if (timing || a.idle_exit_ticks != 0) idle_since = wall_clock64();
      st_batches += 1; st_records += n; st_units += total;
      if (timing) { st_stage += tk1 - tk0; st_resolve += tk2 - tk1; st_write += idle_since - tk2; st_busy += idle_since - tk0; }
      dispatcher_service_pending(a, s, uc);
      if (tracing) {
        counts_dirty = true;
        if (++passes_since_flush >= 256u) {
          for (uint32_t op = tid; op < GPUOS_MAX_OPS; op += kThreads) {
            const uint32_t add = s->opcnt[op];
            if (add) { s->opcnt[op] = 0; __hip_atomic_fetch_add(&a.opcount[op], (uint64_t)add, __ATOMIC_RELAXED, SC_SYSTEM); }
          }
          passes_since_flush = 0;
          counts_dirty = false;
          __syncthreads();
        }
      }
    }
    if (tracing && counts_dirty && mirrored >= tail) {        // the ring ran empty: publish the per-operator counts
      for (uint32_t op = tid; op < GPUOS_MAX_OPS; op += kThreads) {
        const uint32_t add = s->opcnt[op];
        if (add) { s->opcnt[op] = 0; __hip_atomic_fetch_add(&a.opcount[op], (uint64_t)add, __ATOMIC_RELAXED, SC_SYSTEM); }
      }
      passes_since_flush = 0;
      counts_dirty = false;
      __syncthreads();
    }
    if (stopping && mirrored >= tail) {
      while (s->npend != 0) dispatcher_service_pending(a, s, uc);   // nothing is left behind
      drain_stores();                                  // every unit store of every wave has landed ...
      __syncthreads();                                 // ... before the stop flag can be seen
      if (tid == 0) {
        uint64_t* st = a.d->stat;
        // totals over every run of the context's worker
        st[ST_DISP_BATCHES] += st_batches; st[ST_DISP_RECORDS] += st_records; st[ST_DISP_UNITS] += st_units;
        st[ST_DISP_TICKS_STAGE] += st_stage; st[ST_DISP_TICKS_RESOLVE] += st_resolve; st[ST_DISP_TICKS_WRITE] += st_write;
        st[ST_DISP_TICKS_TOTAL_BUSY] += st_busy; st[ST_DISP_POLLS] += polls; st[ST_DISP_DEFERRED] += st_deferred;
        __hip_atomic_store(&a.d->tail_units, uc.w[0], __ATOMIC_RELAXED, SC_SYSTEM);
        __hip_atomic_store(&a.d->tail_units_j, uc.w[1], __ATOMIC_RELAXED, SC_SYSTEM);
        drain_stores();
        __hip_atomic_store(&a.d->stop_dev, 1u, __ATOMIC_RELAXED, SC_SYSTEM);
        __hip_atomic_store(&a.h->exit_code, (ew & 2u) ? 2u : 1u, __ATOMIC_RELAXED, SC_SYSTEM);
      }
      return;
    }
  }
}

union KernelShared {
  DispShared disp;
  WorkShared work;
};

__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(4, 8))) gpuos_worker_kernel(WorkerArgs a) {
  __shared__ KernelShared sh;
  if (blockIdx.x == 0) run_dispatcher(a, &sh.disp);
  else run_worker<0, BuiltinExec>(a, &sh.work);
}

// one ordinary launch per task: block b executes chunk b
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(4, 8))) gpuos_single_task_kernel(Record rec) {
  __shared__ Record s_rec;
  __shared__ alignas(16) float s_red[kScratchFloats];
  if (threadIdx.x == 0) s_rec = rec;
  __syncthreads();
  exec_chunk<POL_PLAIN>(&s_rec, s_rec.impl, blockIdx.x, s_red, nullptr);   // built-in implementations only
}

// The workgroups of a stopped worker left holding work-unit numbers beyond the last published one
// (each claims a number, sees the stop flag and exits): hand those numbers out again, and lower
// the stop flag, before the next worker starts.
__global__ void gpuos_resume_fixup_kernel(DevCtl* d) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    d->claim = d->tail_units;
    d->stop_dev = 0;
  }
}

int launch_resume_fixup(DevCtl* d, void* stream) {
  hipLaunchKernelGGL(gpuos_resume_fixup_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, d);
  return (int)hipGetLastError();
}

// Device-side state (control block, ring mirror, work-unit ring, slot state, operator table) of the
// one context per GPU that gpuos_init_static creates: a file-scope array instead of hipMalloc.  In
// host code the name `scratch` is only a handle for the symbol, not a device address: the address
// on each GPU comes from hipGetSymbolAddress, once per device, with that device current, and that
// pointer is what the host passes on (memset, kernel arguments).
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticScratchBytes];

int static_scratch(int device, void** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptr[kMaxDevices] = {};
  if (device < 0 || device >= kMaxDevices || !out) return (int)hipErrorInvalidValue;
  std::lock_guard<std::mutex> lk(mu);
  if (!ptr[device]) {
    int cur = 0;
    hipError_t e = hipGetDevice(&cur);
    if (e == hipSuccess && cur != device) e = hipSetDevice(device);
    void* p = nullptr;
    if (e == hipSuccess) e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (cur != device) (void)hipSetDevice(cur);
    if (e != hipSuccess) return (int)e;
    if (!p) return (int)hipErrorInvalidSymbol;
    ptr[device] = p;
  }
  *out = ptr[device];
  return (int)hipSuccess;
}

int launch_worker(const WorkerArgs& a, uint32_t grid, void* stream) {
  hipLaunchKernelGGL(gpuos_worker_kernel, dim3(grid), dim3(kThreads), 0, (hipStream_t)stream, a);
  return (int)hipGetLastError();
}

int worker_max_blocks_per_cu(int* out) {
  return (int)hipOccupancyMaxActiveBlocksPerMultiprocessor(out, gpuos_worker_kernel, (int)kThreads, 0);
}

int launch_single(const Record& r, void* stream) {
  const uint32_t grid = r.nchunks ? r.nchunks : 1u;
  hipLaunchKernelGGL(gpuos_single_task_kernel, dim3(grid), dim3(kThreads), 0, (hipStream_t)stream, r);
  return (int)hipGetLastError();
}

}  // namespace gpuos
