// A host thread standing in for the device, for CPU-only tests of the host side of the queue
// protocol (ticket reservation by many producers, wrap-around, back-pressure, check words, the
// doorbell, the dual-slot table, completion harvesting, stop).  TEST INFRASTRUCTURE: it executes
// no operator and touches no tensor; it only speaks the protocol.  The product's host code
// (csrc/gpuos_runtime.cpp) is compiled unchanged against this file, which supplies
//   * the handful of HIP runtime calls the host code makes, on ordinary heap memory, and
//   * launch_worker(): a thread that consumes the ring the way the dispatcher and the workers do
//     (acquire the doorbell, verify each record's check word and ticket, resolve the operator
//     table, write the 8-byte completion words, out of order inside a batch),
// so that the whole thing runs under ThreadSanitizer.
#include <hip/hip_runtime_api.h>

#include <atomic>
#include <chrono>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <random>
#include <thread>

#include "../../include/gpuos.h"
#include "../../paper_2604_17861_amd/csrc/gpuos_internal.h"

namespace {
struct Worker {
  std::thread th;
  std::atomic<bool> done{false};
};
std::mutex g_mu;
std::map<void*, Worker*> g_workers;               // by stream
std::atomic<uint64_t> g_errors{0}, g_records{0}, g_retries{0};
std::atomic<uint64_t> g_alloc_calls{0};             // calls of the allocating / freeing / creating HIP entry points
alignas(256) unsigned char g_scratch[gpuos::kStaticScratchBytes];   // stands in for the library's file-scope device array
// Test hook: the consumer leaves "by itself" (exit code 2, as after an idle time-out) in front of this
// ticket, whatever the doorbell says: the race of an idle exit with a submit, made deterministic.
std::atomic<uint64_t> g_leave_before{~0ull};
// Test hook: the consumer sleeps this long before it serves the next batch (a device that is busy).
std::atomic<uint32_t> g_stall_ms{0};

void consumer(gpuos::WorkerArgs a, Worker* w) {
  using namespace gpuos;
  struct Entry { uint32_t impl = 0, version = 0; } table[GPUOS_MAX_OPS];
  uint64_t mirrored = a.resume_tickets, seen_epoch = 0, polls = 0;      // a worker started again continues the count
  std::mt19937 rng(12345);
  const uint32_t cap = a.cap_mask + 1;
  if (!a.resume) __atomic_store_n(&a.h->clock_origin, 1ull, __ATOMIC_RELEASE);
  while (true) {
    ++polls;
    __atomic_store_n(&a.h->heartbeat, polls, __ATOMIC_RELEASE);
    uint64_t tail = __atomic_load_n(&a.bell->tail, __ATOMIC_ACQUIRE);
    const uint64_t ew = __atomic_load_n(&a.bell->epoch_word, __ATOMIC_ACQUIRE);
    if ((ew >> 12) != (seen_epoch >> 12)) {
      for (uint32_t op = 0; op < GPUOS_MAX_OPS; ++op) {
        const uint32_t ver = __atomic_load_n(&a.htable[op].version, __ATOMIC_ACQUIRE);
        if (ver == 0) continue;
        const uint64_t e = __atomic_load_n(&a.htable[op].slot[ver & 1u], __ATOMIC_RELAXED);
        if ((uint32_t)(e >> 32) != ver) { g_errors.fetch_add(1); continue; }   // the flip came before the slot: a protocol error
        if (ver < table[op].version) g_errors.fetch_add(1);                     // versions only grow
        table[op].impl = (uint32_t)e;
        table[op].version = ver;
      }
    }
    seen_epoch = ew & ~3ull;
    const bool stopping = (ew & 3u) != 0;
    if (stopping) tail = __atomic_load_n(&a.bell->tail, __ATOMIC_ACQUIRE);
    if (tail - mirrored > cap) g_errors.fetch_add(1);                           // the producer overran the ring
    const uint64_t leave = g_leave_before.load();
    if (tail > leave) tail = leave > mirrored ? leave : mirrored;               // ... and does not look at what lies beyond
    while (mirrored < tail) {
      if (const uint32_t ms = g_stall_ms.exchange(0)) std::this_thread::sleep_for(std::chrono::milliseconds(ms));
      const uint32_t n = (uint32_t)((tail - mirrored) < 64 ? (tail - mirrored) : 64);
      uint64_t comp[64];
      for (uint32_t i = 0; i < n; ++i) {
        const uint64_t ticket = mirrored + i;
        Record rec;
        bool good = false;
        for (int attempt = 0; attempt < 1000 && !good; ++attempt) {
          std::memcpy(&rec, &a.hring[ticket & a.cap_mask], sizeof(Record));
          good = record_check_sum(reinterpret_cast<const uint32_t*>(&rec), 64) == record_check_seed(ticket);
          if (!good) g_retries.fetch_add(1);
        }
        int32_t status = GPUOS_OK;
        uint32_t version = 0;
        if (!good || rec.ticket != 0) { g_errors.fetch_add(1); status = GPUOS_E_INVAL; }   // the ticket lives in the check word's seed
        else if (rec.op_id >= GPUOS_MAX_OPS || table[rec.op_id].version == 0) status = GPUOS_E_BADOP;
        else {
          version = table[rec.op_id].version;
          if (table[rec.op_id].impl == GPUOS_IMPL_FAIL) status = GPUOS_E_BADOP;
          if (rec.nchunks == 0 || rec.nchunks > kMaxChunksPerTask) g_errors.fetch_add(1);
        }
        comp[i] = pack_completion(ticket, status, version);
        g_records.fetch_add(1);
      }
      // completions land out of order inside a batch, as they do with a thousand workgroups
      uint32_t order[64];
      for (uint32_t i = 0; i < n; ++i) order[i] = i;
      for (uint32_t i = n; i > 1; --i) std::swap(order[i - 1], order[rng() % i]);
      for (uint32_t k = 0; k < n; ++k) {
        const uint64_t ticket = mirrored + order[k];
        __atomic_store_n(&a.hcomp[ticket & a.cap_mask], comp[order[k]], __ATOMIC_RELEASE);
      }
      mirrored += n;
      __atomic_store_n(&a.h->dispatched, mirrored, __ATOMIC_RELEASE);
    }
    if (stopping && mirrored >= tail) {
      __atomic_store_n(&a.h->exit_code, 1u, __ATOMIC_RELEASE);
      w->done.store(true, std::memory_order_release);
      return;
    }
    if (mirrored >= leave) {
      g_leave_before.store(~0ull);
      __atomic_store_n(&a.h->exit_code, 2u, __ATOMIC_RELEASE);
      w->done.store(true, std::memory_order_release);
      return;
    }
    if ((polls & 15u) == 0) std::this_thread::yield();
  }
}
}  // namespace

extern "C" {
uint64_t standin_errors() { return g_errors.load(); }
uint64_t standin_records() { return g_records.load(); }
uint64_t standin_retries() { return g_retries.load(); }
void standin_leave_before(uint64_t ticket) { g_leave_before.store(ticket); }
void standin_stall_ms(uint32_t ms) { g_stall_ms.store(ms); }
uint64_t standin_alloc_calls() { return g_alloc_calls.load(); }
void standin_scratch_dirty() { std::memset(g_scratch, 0xAB, sizeof(g_scratch)); }     // what a previous context left behind
uint64_t standin_scratch_nonzero(uint64_t n) {
  uint64_t k = 0;
  for (uint64_t i = 0; i < n && i < sizeof(g_scratch); ++i) k += g_scratch[i] != 0;
  return k;
}
}

namespace gpuos {
int launch_worker(const WorkerArgs& a, uint32_t, void* stream) {
  Worker* w = new Worker();
  Worker* old = nullptr;
  {
    std::lock_guard<std::mutex> lk(g_mu);
    auto it = g_workers.find(stream);
    if (it != g_workers.end()) old = it->second;                  // a worker that ran on this stream before and has left
    g_workers[stream] = w;
  }
  if (old) { if (old->th.joinable()) old->th.join(); delete old; }
  w->th = std::thread(consumer, a, w);
  return 0;
}
int launch_resume_fixup(DevCtl* d, void*) { d->claim = d->tail_units; d->stop_dev = 0; return 0; }
int worker_max_blocks_per_cu(int* out) { *out = 4; return 0; }
int launch_single(const Record&, void*) { return 0; }
int static_scratch(int, void** out) { *out = g_scratch; return 0; }
}  // namespace gpuos

// ---- the HIP runtime calls the host code makes, on heap memory -------------------------------
static void* zalloc(size_t n) { void* p = std::aligned_alloc(256, (n + 255) / 256 * 256); if (p) std::memset(p, 0, n); return p; }
hipError_t hipHostMalloc(void** p, size_t n, unsigned int) { g_alloc_calls.fetch_add(1); *p = zalloc(n); return *p ? hipSuccess : hipErrorOutOfMemory; }
hipError_t hipMalloc(void** p, size_t n) { g_alloc_calls.fetch_add(1); *p = zalloc(n); return *p ? hipSuccess : hipErrorOutOfMemory; }
hipError_t hipFree(void* p) { g_alloc_calls.fetch_add(1); std::free(p); return hipSuccess; }
hipError_t hipHostFree(void* p) { g_alloc_calls.fetch_add(1); std::free(p); return hipSuccess; }
hipError_t hipMemset(void* p, int v, size_t n) { std::memset(p, v, n); return hipSuccess; }
hipError_t hipMemsetAsync(void* p, int v, size_t n, hipStream_t) { std::memset(p, v, n); return hipSuccess; }
hipError_t hipMemcpy(void* d, const void* s, size_t n, hipMemcpyKind) { std::memcpy(d, s, n); return hipSuccess; }
hipError_t hipSetDevice(int) { return hipSuccess; }
hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
hipError_t hipGetDeviceProperties(hipDeviceProp_t* p, int) {
  std::memset(p, 0, sizeof(*p));
  p->multiProcessorCount = 4;
  return hipSuccess;
}
hipError_t hipDeviceGetAttribute(int* v, hipDeviceAttribute_t a, int) {       // 4 compute units; no large BAR: host-memory ring
  *v = a == hipDeviceAttributeMultiprocessorCount ? 4 : 0;
  return hipSuccess;
}
hipError_t hipEventCreate(hipEvent_t* e) { g_alloc_calls.fetch_add(1); *e = reinterpret_cast<hipEvent_t>(new int(0)); return hipSuccess; }
hipError_t hipEventDestroy(hipEvent_t e) { delete reinterpret_cast<int*>(e); return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipEventElapsedTime(float* ms, hipEvent_t, hipEvent_t) { *ms = 1.0f; return hipSuccess; }
hipError_t hipStreamCreateWithFlags(hipStream_t* s, unsigned int) { g_alloc_calls.fetch_add(1); *s = reinterpret_cast<hipStream_t>(new int(0)); return hipSuccess; }
hipError_t hipStreamDestroy(hipStream_t s) {
  Worker* w = nullptr;
  {
    std::lock_guard<std::mutex> lk(g_mu);
    auto it = g_workers.find(s);
    if (it != g_workers.end()) { w = it->second; g_workers.erase(it); }
  }
  if (w) { if (w->th.joinable()) w->th.join(); delete w; }
  delete reinterpret_cast<int*>(s);
  return hipSuccess;
}
hipError_t hipStreamQuery(hipStream_t s) {
  std::lock_guard<std::mutex> lk(g_mu);
  auto it = g_workers.find(s);
  if (it == g_workers.end()) return hipSuccess;
  return it->second->done.load(std::memory_order_acquire) ? hipSuccess : hipErrorNotReady;
}
hipError_t hipStreamSynchronize(hipStream_t s) {
  Worker* w = nullptr;
  {
    std::lock_guard<std::mutex> lk(g_mu);
    auto it = g_workers.find(s);
    if (it != g_workers.end()) w = it->second;
  }
  if (w) while (!w->done.load(std::memory_order_acquire)) std::this_thread::yield();
  return hipSuccess;
}
const char* hipGetErrorString(hipError_t) { return "stand-in"; }
// no code objects here: the host code must fall back to interpreted programs
hipError_t hipModuleLoadData(hipModule_t*, const void*) { return hipErrorNotSupported; }
hipError_t hipModuleGetFunction(hipFunction_t*, hipModule_t, const char*) { return hipErrorNotSupported; }
hipError_t hipModuleUnload(hipModule_t) { return hipSuccess; }
hipError_t hipModuleLaunchKernel(hipFunction_t, unsigned int, unsigned int, unsigned int, unsigned int, unsigned int, unsigned int,
                                 unsigned int, hipStream_t, void**, void**) { return hipErrorNotSupported; }
hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t, unsigned int) { return hipSuccess; }
