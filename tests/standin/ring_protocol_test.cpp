// CPU-only test of the host side of the queue protocol against the device stand-in
// (device_standin.cpp), meant to be built with -fsanitize=thread.  Prints one line per check and
// exits non-zero on the first failure.
#include <atomic>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <thread>
#include <vector>

#include <hip/hip_runtime_api.h>

#include "../../include/gpuos.h"
#include "../../paper_2604_17861_amd/csrc/gpuos_internal.h"

extern "C" uint64_t standin_errors();
extern "C" void standin_leave_before(uint64_t ticket);
extern "C" void standin_stall_ms(uint32_t ms);
extern "C" uint64_t standin_records();
extern "C" uint64_t standin_alloc_calls();
extern "C" void standin_scratch_dirty();
extern "C" uint64_t standin_scratch_nonzero(uint64_t n);

#define CHECK(cond) do { if (!(cond)) { std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); std::exit(1); } } while (0)

static gpuos_task add_task(uint16_t op, uint32_t numel, uint16_t dep = 0) {
  gpuos_task t;
  std::memset(&t, 0, sizeof(t));
  t.op_id = op; t.ndim = 1; t.n_inputs = 2; t.size[0] = numel;
  for (int k = 0; k < 2; ++k) { t.in[k].ptr = (void*)(uintptr_t)(0x100000 * (k + 1)); t.in[k].stride[0] = 1; t.in[k].dtype = GPUOS_F32; }
  t.out.ptr = (void*)(uintptr_t)0x900000; t.out.stride[0] = 1; t.out.dtype = GPUOS_F32;
  t.dep[0] = dep;
  return t;
}

static gpuos_ctx* make(uint32_t cap, bool nonblocking = false, bool harvester = false) {
  gpuos_config cfg;
  gpuos_default_config(&cfg);
  cfg.nonblocking_submit = nonblocking;
  cfg.harvester_thread = harvester;
  cfg.wait_timeout_ms = 20000;
  gpuos_ctx* c = nullptr;
  CHECK(gpuos_init(&c, cap, &cfg) == GPUOS_OK);
  CHECK(gpuos_register_op(c, 7, GPUOS_IMPL_ADD, nullptr) == GPUOS_OK);
  CHECK(gpuos_register_op(c, 9, GPUOS_IMPL_MUL, nullptr) == GPUOS_OK);
  return c;
}

// The ring record's check word must reject every mixture of the record a slot held on the previous
// lap and the record being written into it (write-combined stores land piecewise, in any order):
// all 8-byte pieces in which two same-shaped tasks differ, in every old / new combination.
static void check_word_rejects_mixtures() {
  using gpuos::Record;
  auto seal = [](Record& r, uint64_t ticket) {          // what gpuos_submit does to a packed record
    r.ticket = 0;
    r.check = gpuos::record_check_seed(ticket) - gpuos::record_check_sum(reinterpret_cast<const uint32_t*>(&r), 63);
  };
  auto verifies = [](const Record& r, uint64_t ticket) { // what the dispatcher does
    return gpuos::record_check_sum(reinterpret_cast<const uint32_t*>(&r), 64) == gpuos::record_check_seed(ticket);
  };
  for (uint64_t cap : {2ull, 64ull, 4096ull, 65536ull})
    for (uint64_t t : {0ull, 1ull, 63ull, 4095ull, 123456789ull, (1ull << 32) - 1, (1ull << 40) + 17}) {
      Record oldr, newr;
      std::memset(&oldr, 0, sizeof(oldr));
      oldr.op_id = 7; oldr.path = 1; oldr.ndim = 1; oldr.n_inputs = 2; oldr.nchunks = 1; oldr.chunk = 8192; oldr.numel = 2048;
      oldr.size[0] = 2048;
      newr = oldr;
      for (int k = 0; k < 4; ++k) { oldr.ptr[k] = 0x7f0000000000ull + 0x10000000ull * k + 8192ull * 77; newr.ptr[k] = 0x7f0000000000ull + 0x10000000ull * k + 8192ull * 1234; }
      seal(oldr, t);
      seal(newr, t + cap);
      CHECK(verifies(newr, t + cap) && verifies(oldr, t));
      CHECK(!verifies(oldr, t + cap) && !verifies(newr, t));
      const uint64_t* po = reinterpret_cast<const uint64_t*>(&oldr);
      const uint64_t* pn = reinterpret_cast<const uint64_t*>(&newr);
      int diff[32], nd = 0;
      for (int k = 0; k < 32; ++k) if (po[k] != pn[k]) diff[nd++] = k;
      CHECK(nd >= 2 && nd <= 8);
      for (unsigned mask = 0; mask + 1 < (1u << nd); ++mask) {     // every mixture except "all new"
        Record mix = newr;
        uint64_t* pm = reinterpret_cast<uint64_t*>(&mix);
        for (int j = 0; j < nd; ++j) if (!((mask >> j) & 1u)) pm[diff[j]] = po[diff[j]];   // bit clear: the old piece is still there
        CHECK(!verifies(mix, t + cap));
      }
    }
  std::printf("ok: check word rejects every old/new mixture of a slot's records\n");
}

int main() {
  check_word_rejects_mixtures();
  // 1. many producers, tiny rings: every ticket exactly once, consecutive inside a call, in-order log
  for (uint32_t cap : {2u, 8u, 64u}) {
    for (int harv = 0; harv < 2; ++harv) {
      gpuos_ctx* c = make(cap, false, harv != 0);
      const int n_threads = 6, per_thread = 3000;
      std::vector<std::vector<uint64_t>> firsts(n_threads);
      std::vector<std::thread> th;
      std::atomic<int> failures{0};
      for (int k = 0; k < n_threads; ++k)
        th.emplace_back([&, k] {
          unsigned s = 17u * (unsigned)k + 1u;
          int left = per_thread;
          while (left > 0) {
            s = s * 1664525u + 1013904223u;
            int m = 1 + (int)((s >> 16) % 5u);
            if (m > left) m = left;
            gpuos_task batch[5];
            for (int i = 0; i < m; ++i) batch[i] = add_task(k % 2 ? 7 : 9, 1000 + (uint32_t)i, i > 0 ? 1 : 0);   // chain inside the call
            uint64_t first = ~0ull;
            // (every third call as submit + flush in one: records and doorbell leave with one flush)
            const int rc = (s >> 4) % 3u == 0 ? gpuos_submit_flush(c, batch, (uint32_t)m, &first) : gpuos_submit(c, batch, (uint32_t)m, &first);
            if (rc != GPUOS_OK) { failures++; return; }
            for (int i = 0; i < m; ++i) firsts[k].push_back(first + (uint64_t)i);
            if ((s >> 8) % 7u == 0 && gpuos_wait(c, first + (uint64_t)m - 1, 0) != GPUOS_OK) { failures++; return; }
            if ((s >> 8) % 11u == 0) gpuos_flush(c);
            left -= m;
          }
        });
      for (auto& t : th) t.join();
      CHECK(failures.load() == 0);
      CHECK(gpuos_wait(c, GPUOS_ALL, 0) == GPUOS_OK);
      const uint64_t total = (uint64_t)n_threads * per_thread;
      std::vector<int> seen(total, 0);
      for (auto& v : firsts) for (uint64_t t : v) { CHECK(t < total); seen[t]++; }
      for (uint64_t t = 0; t < total; ++t) CHECK(seen[t] == 1);
      std::vector<gpuos_completion> comp(total);
      CHECK(gpuos_get_completions(c, 0, (uint32_t)total, comp.data()) == GPUOS_OK);
      for (uint64_t t = 0; t < total; ++t) {
        CHECK(comp[t].ticket == t && comp[t].status == 0 && comp[t].op_version == 1);
        CHECK(comp[t].t_done_ns >= comp[t].t_submit_ns);
      }
      gpuos_queue_state q;
      CHECK(gpuos_peek_queue(c, &q) == GPUOS_OK);
      CHECK(q.head_submitted == total && q.tail_published == total && q.claimed == total && q.completed == total);
      CHECK(gpuos_worker_alive(c) == 1);
      CHECK(gpuos_shutdown(c) == GPUOS_OK);
      std::printf("ok: %d producers x %d tasks, capacity %u, harvester thread %d\n", n_threads, per_thread, cap, harv);
    }
  }
  // 2. a full ring in non-blocking mode: E_FULL and nothing enqueued; a dependency that reaches
  //    before the first ticket or beyond the ring is rejected
  {
    gpuos_ctx* c = make(4, true);
    gpuos_task five[5];
    for (int i = 0; i < 5; ++i) five[i] = add_task(7, 64);
    uint64_t first = 0;
    CHECK(gpuos_submit(c, five, 5, &first) == GPUOS_E_FULL);
    gpuos_queue_state q;
    CHECK(gpuos_peek_queue(c, &q) == GPUOS_OK && q.head_submitted == 0);
    gpuos_task bad = add_task(7, 64, 1);
    CHECK(gpuos_submit(c, &bad, 1, nullptr) == GPUOS_E_INVAL);          // ticket 0 has nothing before it
    CHECK(gpuos_submit(c, five, 4, &first) == GPUOS_OK && first == 0);
    CHECK(gpuos_wait(c, GPUOS_ALL, 0) == GPUOS_OK);
    bad = add_task(7, 64, 4);
    CHECK(gpuos_submit(c, &bad, 1, nullptr) == GPUOS_E_INVAL);          // back-distance >= capacity
    bad = add_task(200, 64);
    CHECK(gpuos_submit(c, &bad, 1, nullptr) == GPUOS_E_BADOP);          // never registered
    CHECK(gpuos_shutdown(c) == GPUOS_OK);
    std::printf("ok: non-blocking ring, dependency and op-id checks\n");
  }
  // 3. swaps while producers run: versions never go back in ticket order, the kill switch shows,
  //    a swap returns only versions that later tasks observe
  {
    gpuos_ctx* c = make(16);
    std::atomic<bool> stop{false};
    std::atomic<uint64_t> after_swap_first{0};
    std::thread prod([&] {
      gpuos_task t = add_task(7, 128);
      while (!stop.load()) CHECK(gpuos_submit(c, &t, 1, nullptr) == GPUOS_OK);
    });
    uint32_t v = 0;
    for (int i = 0; i < 40; ++i) {
      CHECK(gpuos_swap_op(c, 7, i % 2 ? GPUOS_IMPL_ADD : GPUOS_IMPL_SUB, &v) == GPUOS_OK);
      CHECK(v == (uint32_t)i + 2);
    }
    CHECK(gpuos_swap_op(c, 7, GPUOS_IMPL_RELU, &v) == GPUOS_E_INVAL);   // arity differs
    stop.store(true);
    prod.join();
    gpuos_task t = add_task(7, 128);
    uint64_t tk = 0;
    CHECK(gpuos_submit(c, &t, 1, &tk) == GPUOS_OK);
    CHECK(gpuos_wait(c, tk, 0) == GPUOS_OK);
    std::vector<gpuos_completion> comp(tk + 1);
    // the log holds at least the last 2^20 tickets
    const uint64_t lo = tk + 1 > (1u << 20) ? tk + 1 - (1u << 20) : 0;
    CHECK(gpuos_get_completions(c, lo, (uint32_t)(tk + 1 - lo), comp.data()) == GPUOS_OK);
    for (uint64_t i = 1; i + lo <= tk; ++i) CHECK(comp[i].op_version >= comp[i - 1].op_version);
    CHECK(comp[tk - lo].op_version == 41);
    CHECK(gpuos_kill_op(c, 7, &v) == GPUOS_OK && v == 42);
    CHECK(gpuos_submit(c, &t, 1, &tk) == GPUOS_OK);
    CHECK(gpuos_wait(c, tk, 0) == GPUOS_E_BADOP);
    CHECK(gpuos_wait(c, GPUOS_ALL, 0) == GPUOS_E_BADOP);                // first error, reported once
    CHECK(gpuos_wait(c, GPUOS_ALL, 0) == GPUOS_OK);
    // the audit log has every change, in order: one register (make()), 40 swaps, the kill
    uint64_t total = 0;
    CHECK(gpuos_audit_log(c, 0, 0, nullptr, &total) == GPUOS_OK);
    std::vector<gpuos_audit_record> log(total);
    CHECK(gpuos_audit_log(c, 0, (uint32_t)total, log.data(), nullptr) == GPUOS_OK);
    CHECK(gpuos_audit_log(c, 1, (uint32_t)total, log.data(), nullptr) == GPUOS_E_INVAL);
    size_t swaps = 0, kills = 0, regs = 0;
    uint32_t last_v = 0;
    for (size_t i = 0; i < log.size(); ++i) {
      if (i) CHECK(log[i].t_ns >= log[i - 1].t_ns && log[i].head_ticket >= log[i - 1].head_ticket);
      if (log[i].op_id != 7) { regs += log[i].kind == GPUOS_AUDIT_REGISTER; continue; }
      CHECK(log[i].version == last_v + 1);
      last_v = log[i].version;
      if (log[i].kind == GPUOS_AUDIT_REGISTER) { regs++; CHECK(log[i].version == 1 && log[i].head_ticket == 0); }
      else if (log[i].kind == GPUOS_AUDIT_SWAP) { swaps++; CHECK(log[i].impl_id == (log[i].version % 2 ? GPUOS_IMPL_ADD : GPUOS_IMPL_SUB)); }
      else if (log[i].kind == GPUOS_AUDIT_KILL) { kills++; CHECK(log[i].impl_id == GPUOS_IMPL_FAIL && log[i].version == 42 && log[i].head_ticket == tk); }
    }
    CHECK(swaps == 40 && kills == 1 && regs >= 1 && last_v == 42);
    CHECK(gpuos_shutdown(c) == GPUOS_OK);
    std::printf("ok: 40 swaps under load, kill switch, audit log\n");
  }
  // 4. shutdown with tasks in flight drains them; use after stop is refused; programs are table entries
  {
    gpuos_ctx* c = make(32);
    gpuos_instr code[2] = {{GPUOS_PC_ADD, 0, 0, 1, 0.f}, {GPUOS_PC_MUL, 0, 0, 3, 0.f}};
    uint32_t impl = 0;
    CHECK(gpuos_define_program(c, code, 2, 2, &impl) == GPUOS_OK && impl == GPUOS_IMPL_PROGRAM_BASE);
    CHECK(gpuos_register_op(c, 30, impl, nullptr) == GPUOS_OK);
    CHECK(gpuos_register_op(c, 31, impl + 1, nullptr) == GPUOS_E_BADOP);
    {
      uint64_t total = 0;
      CHECK(gpuos_audit_log(c, 0, 0, nullptr, &total) == GPUOS_OK && total >= 2);
      gpuos_audit_record two[2];
      CHECK(gpuos_audit_log(c, total - 2, 2, two, nullptr) == GPUOS_OK);
      uint64_t h = 0xcbf29ce484222325ull;
      for (size_t b = 0; b < sizeof(code); ++b) h = (h ^ reinterpret_cast<const unsigned char*>(code)[b]) * 0x100000001b3ull;
      CHECK(two[0].kind == GPUOS_AUDIT_DEFINE_PROGRAM && two[0].impl_id == impl && two[0].n_instr == 2 && two[0].n_inputs == 2 && two[0].code_hash == h);
      CHECK(two[1].kind == GPUOS_AUDIT_REGISTER && two[1].op_id == 30 && two[1].impl_id == impl && two[1].code_hash == h && two[1].version == 1);
    }
    code[1].a = 9;
    CHECK(gpuos_define_program(c, code, 2, 2, &impl) == GPUOS_E_INVAL);
    std::vector<gpuos_task> many(500, add_task(30, 4096));
    CHECK(gpuos_submit(c, many.data(), 500, nullptr) == GPUOS_OK);
    CHECK(gpuos_stop_worker(c) == GPUOS_OK);
    gpuos_queue_state q;
    CHECK(gpuos_peek_queue(c, &q) == GPUOS_OK && q.completed == 500);
    CHECK(gpuos_submit(c, many.data(), 1, nullptr) == GPUOS_E_DEAD);
    CHECK(gpuos_worker_alive(c) == 0);
    CHECK(gpuos_shutdown(c) == GPUOS_OK);
    std::printf("ok: shutdown drains, use after stop refused, program ids\n");
  }
  // 5. the worker stopped and started again several times: tickets, the completion log, the
  //    operator table (a swap made while stopped) and the ring position all continue
  for (int harv = 0; harv < 2; ++harv) {
    gpuos_ctx* c = make(8, false, harv != 0);
    uint64_t expect = 0;
    uint32_t v = 0;
    for (int round = 0; round < 5; ++round) {
      std::vector<gpuos_task> some(13 + 7 * round, add_task(7, 256));
      uint64_t first = ~0ull;
      CHECK(gpuos_submit(c, some.data(), (uint32_t)some.size(), &first) == GPUOS_OK && first == expect);
      expect += some.size();
      CHECK(gpuos_start_worker(c) == GPUOS_OK);                          // running: nothing to do
      CHECK(gpuos_stop_worker(c) == GPUOS_OK);                           // drains
      gpuos_queue_state q;
      CHECK(gpuos_peek_queue(c, &q) == GPUOS_OK && q.completed == expect && q.claimed == expect);
      CHECK(gpuos_worker_alive(c) == 0);
      CHECK(gpuos_submit(c, some.data(), 1, nullptr) == GPUOS_E_DEAD);
      CHECK(gpuos_swap_op(c, 7, round % 2 ? GPUOS_IMPL_ADD : GPUOS_IMPL_SUB, &v) == GPUOS_OK && v == (uint32_t)round + 2);
      CHECK(gpuos_start_worker(c) == GPUOS_OK);
      CHECK(gpuos_worker_alive(c) == 1);
      uint64_t tk = 0;
      CHECK(gpuos_submit(c, some.data(), 1, &tk) == GPUOS_OK && tk == expect);
      expect += 1;
      CHECK(gpuos_wait(c, tk, 0) == GPUOS_OK);
      gpuos_completion comp;
      CHECK(gpuos_get_completions(c, tk, 1, &comp) == GPUOS_OK && comp.ticket == tk && comp.op_version == (uint32_t)round + 2);
    }
    CHECK(gpuos_shutdown(c) == GPUOS_OK);
    std::printf("ok: worker stopped and started 5 times, harvester thread %d\n", harv);
  }
  // 5b. an idle exit that races with a submit: the worker leaves without having seen the last
  //     doorbell; the wait says so, and the worker started again executes what was left in the ring
  {
    gpuos_ctx* c = make(16);
    std::vector<gpuos_task> some(10, add_task(7, 256));
    uint64_t tk = 0;
    CHECK(gpuos_submit(c, some.data(), 4, &tk) == GPUOS_OK && tk == 0);
    CHECK(gpuos_wait(c, 3, 0) == GPUOS_OK);
    standin_leave_before(6);                                          // tickets 4, 5 will be served, 6.. not
    CHECK(gpuos_submit(c, some.data(), 10, &tk) == GPUOS_OK && tk == 4);
    CHECK(gpuos_wait(c, 5, 0) == GPUOS_OK);
    CHECK(gpuos_wait(c, GPUOS_ALL, 0) == GPUOS_E_DEAD);
    CHECK(gpuos_worker_alive(c) == 0);
    gpuos_queue_state q;
    CHECK(gpuos_peek_queue(c, &q) == GPUOS_OK && q.completed == 6 && q.claimed == 6 && q.head_submitted == 14);
    CHECK(gpuos_start_worker(c) == GPUOS_OK);
    CHECK(gpuos_wait(c, GPUOS_ALL, 0) == GPUOS_OK);
    CHECK(gpuos_peek_queue(c, &q) == GPUOS_OK && q.completed == 14 && q.claimed == 14);
    std::vector<gpuos_completion> comp(14);
    CHECK(gpuos_get_completions(c, 0, 14, comp.data()) == GPUOS_OK);
    for (uint64_t t = 0; t < 14; ++t) CHECK(comp[t].ticket == t && comp[t].status == 0);
    CHECK(gpuos_submit(c, some.data(), 3, &tk) == GPUOS_OK && tk == 14);
    CHECK(gpuos_wait(c, GPUOS_ALL, 0) == GPUOS_OK);
    CHECK(gpuos_shutdown(c) == GPUOS_OK);
    std::printf("ok: tasks stranded by an idle exit are executed after a restart\n");
  }
  // 5c. a wait with a time limit on a device that is busy: GPUOS_E_TIMEOUT, nothing lost, the same
  //     wait without a limit succeeds; a ticket that was never issued is refused
  {
    gpuos_ctx* c = make(16);
    gpuos_task t = add_task(7, 256);
    uint64_t tk = 0;
    standin_stall_ms(400);
    CHECK(gpuos_submit(c, &t, 1, &tk) == GPUOS_OK);
    const auto t0 = std::chrono::steady_clock::now();
    CHECK(gpuos_wait(c, tk, 30ull * 1000 * 1000) == GPUOS_E_TIMEOUT);
    const double waited = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    CHECK(waited > 0.025 && waited < 0.3);
    CHECK(gpuos_worker_alive(c) == 1);
    CHECK(gpuos_wait(c, tk + 1, 0) == GPUOS_E_INVAL);
    CHECK(gpuos_wait(c, tk, 0) == GPUOS_OK);
    CHECK(gpuos_wait(c, GPUOS_ALL, 1) == GPUOS_OK);                     // complete already: no time is needed
    CHECK(gpuos_shutdown(c) == GPUOS_OK);
    std::printf("ok: wait with a time limit\n");
  }
  // 5d. back-pressure that runs into the time limit in the middle of a submit: the records written
  //     before the stall keep their tickets and are executed, the rest were never submitted, and
  //     the next submit continues right after them
  {
    gpuos_config cfg;
    gpuos_default_config(&cfg);
    cfg.wait_timeout_ms = 400;
    gpuos_ctx* c = nullptr;
    CHECK(gpuos_init(&c, 16, &cfg) == GPUOS_OK);
    CHECK(gpuos_register_op(c, 7, GPUOS_IMPL_ADD, nullptr) == GPUOS_OK);
    std::vector<gpuos_task> many(40, add_task(7, 256));
    uint64_t tk = ~0ull;
    standin_stall_ms(1600);
    CHECK(gpuos_submit(c, many.data(), 40, &tk) == GPUOS_E_TIMEOUT);
    CHECK(tk == 0);
    gpuos_queue_state q;
    CHECK(gpuos_peek_queue(c, &q) == GPUOS_OK);
    const uint64_t taken = q.head_submitted - tk;
    CHECK(taken == 16);                                                 // one ring's worth went in before the ring was full
    CHECK(gpuos_wait(c, GPUOS_ALL, 5000ull * 1000 * 1000) == GPUOS_OK);
    std::vector<gpuos_completion> comp(taken);
    CHECK(gpuos_get_completions(c, 0, (uint32_t)taken, comp.data()) == GPUOS_OK);
    for (uint64_t t = 0; t < taken; ++t) CHECK(comp[t].ticket == t && comp[t].status == 0);
    CHECK(gpuos_submit(c, many.data(), 3, &tk) == GPUOS_OK && tk == taken);
    CHECK(gpuos_wait(c, GPUOS_ALL, 5000ull * 1000 * 1000) == GPUOS_OK);
    CHECK(gpuos_shutdown(c) == GPUOS_OK);
    std::printf("ok: a submit that times out under back-pressure keeps what it had written\n");
  }
  // 6. profiler markers: with cfg.markers the calls are annotated through the marker library the
  //    environment names (the test driver points it at a recorder); off by default
  if (std::getenv("GPUOS_ROCTX_LIBRARY")) {
    gpuos_config cfg;
    gpuos_default_config(&cfg);
    CHECK(cfg.markers == 0);
    cfg.markers = 1;
    cfg.wait_timeout_ms = 20000;
    gpuos_ctx* c = nullptr;
    CHECK(gpuos_init(&c, 16, &cfg) == GPUOS_OK);
    uint32_t v = 0;
    CHECK(gpuos_register_op(c, 7, GPUOS_IMPL_ADD, &v) == GPUOS_OK);
    std::vector<gpuos_task> some(5, add_task(7, 256));
    uint64_t tk = 0;
    CHECK(gpuos_submit(c, some.data(), 5, &tk) == GPUOS_OK);
    CHECK(gpuos_wait(c, tk + 4, 0) == GPUOS_OK);
    CHECK(gpuos_swap_op(c, 7, GPUOS_IMPL_SUB, &v) == GPUOS_OK);
    CHECK(gpuos_stop_worker(c) == GPUOS_OK);
    CHECK(gpuos_start_worker(c) == GPUOS_OK);
    CHECK(gpuos_wait(c, GPUOS_ALL, 0) == GPUOS_OK);
    CHECK(gpuos_shutdown(c) == GPUOS_OK);
    std::printf("ok: markers\n");
  }
  // 7. the context that allocates nothing: device-side state in the library's static array, host side
  //    in the caller's block, the caller's stream; one such context per device at a time; the array
  //    is cleared of what the previous context left
  {
    gpuos_config cfg;
    gpuos_default_config(&cfg);
    cfg.wait_timeout_ms = 20000;
    const uint64_t bytes = GPUOS_STATIC_HOST_BYTES(GPUOS_STATIC_MAX_CAPACITY);
    void* block = std::aligned_alloc(256, bytes);
    void* block2 = std::aligned_alloc(256, bytes);
    CHECK(block && block2);
    std::memset(block, 0x5A, bytes);
    hipStream_t st1 = nullptr, st2 = nullptr;
    CHECK(hipStreamCreateWithFlags(&st1, 0) == hipSuccess && hipStreamCreateWithFlags(&st2, 0) == hipSuccess);
    gpuos_ctx* c = nullptr;
    gpuos_ctx* c2 = nullptr;
    CHECK(gpuos_init_static(&c, 2048, &cfg, block, bytes, st1) == GPUOS_E_INVAL && c == nullptr);        // beyond the maximum
    CHECK(std::strstr(gpuos_last_hip_error(), "GPUOS_STATIC_MAX_CAPACITY") != nullptr);
    CHECK(gpuos_init_static(&c, 64, &cfg, block, 1000, st1) == GPUOS_E_INVAL);                           // block too small
    CHECK(gpuos_init_static(&c, 64, &cfg, (char*)block + 8, bytes - 8, st1) == GPUOS_E_INVAL);           // misaligned
    CHECK(gpuos_init_static(&c, 64, &cfg, block, bytes, nullptr) == GPUOS_E_INVAL);                      // no stream
    for (uint32_t cap : {64u, 16u}) {                                                                   // twice in a row, the second one smaller
      standin_scratch_dirty();
      const uint64_t a0 = standin_alloc_calls();
      CHECK(gpuos_init_static(&c, cap, &cfg, block, bytes, st1) == GPUOS_OK && c != nullptr);
      CHECK(standin_alloc_calls() == a0);                                                                // no hipMalloc / hipHostMalloc / stream / event
      CHECK(standin_scratch_nonzero(gpuos::static_layout(cap).total) == 0);                              // what the last context left is gone
      CHECK(gpuos_init_static(&c2, 16, &cfg, block2, bytes, st2) == GPUOS_E_FULL && c2 == nullptr);      // one at a time per device
      CHECK(gpuos_register_op(c, 7, GPUOS_IMPL_ADD, nullptr) == GPUOS_OK);
      std::vector<gpuos_task> some(200, add_task(7, 256));
      uint64_t tk = 0;
      CHECK(gpuos_submit(c, some.data(), 200, &tk) == GPUOS_OK && tk == 0);                              // wraps the ring several times
      CHECK(gpuos_wait(c, GPUOS_ALL, 0) == GPUOS_OK);
      std::vector<gpuos_completion> comp(cap);
      CHECK(gpuos_get_completions(c, 200 - cap, cap, comp.data()) == GPUOS_OK);
      for (uint32_t t = 0; t < cap; ++t) CHECK(comp[t].ticket == 200 - cap + t && comp[t].status == 0 && comp[t].op_version == 1);
      gpuos_queue_state q;
      CHECK(gpuos_peek_queue(c, &q) == GPUOS_OK && q.capacity == cap && q.push_ring == 0 && q.completed == 200);
      CHECK(gpuos_stop_worker(c) == GPUOS_OK);
      float ms = 0;
      CHECK(gpuos_worker_elapsed_ms(c, &ms) == GPUOS_E_INVAL);                                           // no events on such a context
      CHECK(gpuos_start_worker(c) == GPUOS_OK);
      CHECK(gpuos_submit(c, some.data(), 5, &tk) == GPUOS_OK && tk == 200);
      CHECK(gpuos_wait(c, GPUOS_ALL, 0) == GPUOS_OK);
      const uint64_t a1 = standin_alloc_calls();
      CHECK(gpuos_shutdown(c) == GPUOS_OK);
      CHECK(standin_alloc_calls() == a1);                                                                // ... and nothing is freed that was not allocated
      c = nullptr;
    }
    CHECK(hipStreamDestroy(st1) == hipSuccess && hipStreamDestroy(st2) == hipSuccess);
    std::free(block); std::free(block2);
    std::printf("ok: a context that allocates nothing, twice in a row\n");
  }
  CHECK(standin_errors() == 0);
  std::printf("all ok: %llu records through the stand-in, 0 protocol errors\n", (unsigned long long)standin_records());
  return 0;
}
