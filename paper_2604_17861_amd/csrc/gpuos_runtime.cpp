// gpuos_runtime.cpp -- host side of the GPUOS hot path: the C ABI of
// include/gpuos.h.  Descriptor validation / coalescing / packing, the ring
// producer (paper Section 4.2: acquire slot, write, commit with a store-release),
// completion harvesting, the dual-slot operator table (Section 4.1) and the
// lifecycle of the persistent worker (Section 5.4 / Table 1).

#include <hip/hip_runtime_api.h>

#include <atomic>
#include <chrono>
#include <cstddef>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include <immintrin.h>
#include <dlfcn.h>
#include <pthread.h>
#include <sched.h>

#include "../../include/gpuos.h"
#include "gpuos_internal.h"

using namespace gpuos;

namespace gpuos {        // csrc/gpuos_jit.cpp: operator programs -> code object of the run-time worker kernel
bool jit_compiler_available();
int jit_build(const ProgramImage* imgs, uint32_t n, std::vector<char>* code, std::string* err, double* compile_ms, bool* cache_hit);
void jit_cache_counts(uint64_t* compiles, uint64_t* hits);
}

namespace {

thread_local std::string g_hip_error;

bool hip_ok(hipError_t e, const char* what) {
  if (e == hipSuccess) return true;
  g_hip_error = std::string(what) + ": " + hipGetErrorString(e);
  return false;
}
#define HIP_TRY(call) do { if (!hip_ok((call), #call)) return GPUOS_E_HIP; } while (0)

// Profiler markers (paper Section 5.3: markers a timeline tool shows next to the kernels).  The
// roctx entry points are looked up once, at the first use, in the profiler SDK's library or the
// older one; a process that is not being profiled pays a null check.
struct Roctx {
  int (*push)(const char*) = nullptr;
  int (*pop)() = nullptr;
  void (*mark)(const char*) = nullptr;
};
const Roctx& roctx() {
  static const Roctx r = [] {
    Roctx x;
    const char* names[3] = {std::getenv("GPUOS_ROCTX_LIBRARY"), "librocprofiler-sdk-roctx.so.1", "libroctx64.so.4"};
    for (const char* n : names) {
      if (!n || !*n) continue;
      void* h = dlopen(n, RTLD_NOW | RTLD_GLOBAL);
      if (!h) continue;
      x.push = reinterpret_cast<int (*)(const char*)>(dlsym(h, "roctxRangePushA"));
      x.pop = reinterpret_cast<int (*)()>(dlsym(h, "roctxRangePop"));
      x.mark = reinterpret_cast<void (*)(const char*)>(dlsym(h, "roctxMarkA"));
      if (x.push && x.pop && x.mark) break;
      x = Roctx();
    }
    return x;
  }();
  return r;
}
struct MarkerRange {                    // a range on the calling thread for the lifetime of the object
  bool on;
  MarkerRange(bool enabled, const char* fmt, unsigned long long a = 0, unsigned long long b = 0) : on(enabled && roctx().push) {
    if (!on) return;
    char buf[96];
    std::snprintf(buf, sizeof(buf), fmt, a, b);
    roctx().push(buf);
  }
  ~MarkerRange() { if (on) roctx().pop(); }
};
void marker(bool enabled, const char* fmt, unsigned long long a = 0, unsigned long long b = 0, unsigned long long c3 = 0) {
  if (!enabled || !roctx().mark) return;
  char buf[96];
  std::snprintf(buf, sizeof(buf), fmt, a, b, c3);
  roctx().mark(buf);
}

// The producers' lock.  It is held for a few microseconds at a time (the ring writes of one batch),
// and a waiter is usually the next producer with its batch already packed: spin on the flag first
// (test-and-test-and-set with pause), and only give the time slice away when that takes long (the
// holder lost its core, or waits for room in a full ring).  A futex-based mutex puts waiters to
// sleep after a few hundred nanoseconds and pays a wake-up on every hand-over.
class SpinMutex {
 public:
  void lock() {
    for (uint32_t spins = 0;; ++spins) {
      if (!flag_.load(std::memory_order_relaxed) && !flag_.exchange(true, std::memory_order_acquire)) return;
      if (spins < 4096) __builtin_ia32_pause();
      else sched_yield();
    }
  }
  bool try_lock() { return !flag_.load(std::memory_order_relaxed) && !flag_.exchange(true, std::memory_order_acquire); }
  void unlock() { flag_.store(false, std::memory_order_release); }
 private:
  std::atomic<bool> flag_{false};
};

inline uint64_t now_ns() {
  return (uint64_t)std::chrono::duration_cast<std::chrono::nanoseconds>(
             std::chrono::steady_clock::now().time_since_epoch()).count();
}

// ---- static facts about the implementations -------------------------------------
int impl_arity(uint32_t impl) {
  switch (impl) {
    case GPUOS_IMPL_ADD: case GPUOS_IMPL_SUB: case GPUOS_IMPL_MUL: case GPUOS_IMPL_DIV:
    case GPUOS_IMPL_SUB_EXP: return 2;
    case GPUOS_IMPL_FMA: return 3;
    case GPUOS_IMPL_RELU: case GPUOS_IMPL_EXP: case GPUOS_IMPL_GELU_ERF: case GPUOS_IMPL_GELU_TANH:
    case GPUOS_IMPL_SCALE: case GPUOS_IMPL_COPY: case GPUOS_IMPL_SUM_LAST: case GPUOS_IMPL_MAX_LAST:
    case GPUOS_IMPL_MIN_LAST: case GPUOS_IMPL_SOFTMAX_LAST: return 1;
    case GPUOS_IMPL_MASKED_SOFTMAX_LAST: return 2;
    case GPUOS_IMPL_LAYERNORM_LAST: return 3;
    default: return -1;
  }
}
bool impl_is_reduction(uint32_t impl) {
  return impl == GPUOS_IMPL_SUM_LAST || impl == GPUOS_IMPL_MAX_LAST || impl == GPUOS_IMPL_MIN_LAST;
}
bool impl_is_rowop(uint32_t impl) {
  return impl == GPUOS_IMPL_SOFTMAX_LAST || impl == GPUOS_IMPL_MASKED_SOFTMAX_LAST || impl == GPUOS_IMPL_LAYERNORM_LAST;
}
int impl_kind(uint32_t impl) { return impl_is_reduction(impl) ? 1 : (impl_is_rowop(impl) ? 2 : 0); }
bool impl_takes_int(uint32_t impl) {
  return impl == GPUOS_IMPL_ADD || impl == GPUOS_IMPL_SUB || impl == GPUOS_IMPL_MUL ||
         impl == GPUOS_IMPL_COPY || impl_is_reduction(impl);
}
inline uint32_t dtype_size(uint32_t dt) { return (dt == GPUOS_F32 || dt == GPUOS_I32) ? 4u : 2u; }

constexpr int64_t kMaxExtent = 2147483647LL;

struct Operand {              // one tensor after masking broadcast dims
  uint64_t ptr;
  int64_t stride[GPUOS_MAX_DIMS];
  uint32_t dtype;
};

int check_operand(const gpuos_tensor& t, int ndim, const int64_t* size, bool is_out, Operand* o) {
  if (t.ptr == nullptr || t.dtype > GPUOS_I32) return GPUOS_E_INVAL;
  if ((uint64_t)t.ptr % dtype_size(t.dtype) != 0) return GPUOS_E_INVAL;   // elements are naturally aligned
  if (is_out && t.bcast_mask != 0) return GPUOS_E_INVAL;
  int64_t max_off = 0;
  o->ptr = (uint64_t)t.ptr;
  o->dtype = t.dtype;
  for (int d = 0; d < GPUOS_MAX_DIMS; ++d) o->stride[d] = 0;
  for (int d = 0; d < ndim; ++d) {
    if (t.stride[d] < 0) return GPUOS_E_INVAL;
    const int64_t s = ((t.bcast_mask >> d) & 1) ? 0 : t.stride[d];
    if (size[d] > 1) {
      if (is_out && s == 0) return GPUOS_E_INVAL;        // output would overlap itself
      if (s > kMaxExtent) return GPUOS_E_INVAL;
      max_off += (size[d] - 1) * s;
      if (max_off > kMaxExtent) return GPUOS_E_INVAL;
      o->stride[d] = s;
    }
  }
  return GPUOS_OK;
}

// Merge adjacent dims that every operand walks as one: outer stride == inner
// stride * inner size for all operands.  Size-1 dims are dropped first.
int coalesce(int nd, int64_t* size, Operand* ops, int nops) {
  int64_t sz[GPUOS_MAX_DIMS];
  int64_t st[5][GPUOS_MAX_DIMS];
  int m = 0;
  for (int d = 0; d < nd; ++d) {
    if (size[d] == 1) continue;
    sz[m] = size[d];
    for (int k = 0; k < nops; ++k) st[k][m] = ops[k].stride[d];
    ++m;
  }
  if (m == 0) {                                   // a single element
    sz[0] = 1;
    for (int k = 0; k < nops; ++k) st[k][0] = 1;
    m = 1;
  }
  int w = 0;                                      // index of the dim being grown (outermost so far)
  for (int d = 1; d < m; ++d) {
    bool merge = true;
    for (int k = 0; k < nops; ++k)
      if (st[k][w] != st[k][d] * sz[d]) { merge = false; break; }
    if (merge) {
      sz[w] *= sz[d];
      for (int k = 0; k < nops; ++k) st[k][w] = st[k][d];
    } else {
      ++w;
      sz[w] = sz[d];
      for (int k = 0; k < nops; ++k) st[k][w] = st[k][d];
    }
  }
  m = w + 1;
  for (int d = 0; d < GPUOS_MAX_DIMS; ++d) {
    size[d] = d < m ? sz[d] : 1;
    for (int k = 0; k < nops; ++k) ops[k].stride[d] = d < m ? st[k][d] : 0;
  }
  return m;
}

inline bool aligned16(uint64_t p) { return (p & 15u) == 0; }

// Validate `t` for implementation `impl` and pack it.  Nothing is written to
// *r unless the result is GPUOS_OK.
int pack_task(const gpuos_task& t, uint32_t impl, Record* r, uint32_t chunk_elems = kChunkElems, int program_arity = 0) {
  Record rec;
  std::memset(&rec, 0, sizeof(rec));
  rec.op_id = t.op_id;
  rec.alpha = t.alpha;
  rec.impl = impl;
  rec.dep[0] = t.dep[0]; rec.dep[1] = t.dep[1]; rec.dep[2] = t.dep[2];
  if (t.flags & ~(GPUOS_FLAG_FENCE | GPUOS_FLAG_KEEPDIM)) return GPUOS_E_INVAL;
  if (t.flags & GPUOS_FLAG_FENCE) rec.rflags |= RF_FENCE;
  if (impl == GPUOS_IMPL_FAIL) {                   // executes nothing; one unit reports it
    rec.path = PATH_NOP;
    rec.nchunks = 1;
    *r = rec;
    return GPUOS_OK;
  }
  // an operator program: elementwise, float-only, the arity it was defined with
  const int ar = impl >= GPUOS_IMPL_PROGRAM_BASE ? (program_arity > 0 ? program_arity : -1) : impl_arity(impl);
  if (ar < 0) return GPUOS_E_BADOP;
  if (t.ndim < 1 || t.ndim > GPUOS_MAX_DIMS || t.n_inputs != ar) return GPUOS_E_INVAL;
  int64_t size[GPUOS_MAX_DIMS];
  int64_t numel = 1;
  for (int d = 0; d < GPUOS_MAX_DIMS; ++d) size[d] = 1;
  for (int d = 0; d < t.ndim; ++d) {
    if (t.size[d] < 0 || t.size[d] > kMaxExtent) return GPUOS_E_INVAL;
    size[d] = t.size[d];
    numel *= size[d];
    if (numel > kMaxExtent) return GPUOS_E_INVAL;
  }
  // Chunk size: chunk_elems (about 192 KiB of traffic) streams best for the largest tensors; tasks
  // of up to a million elements are split twice as finely, which shortens the critical path of
  // dependent chains of mid-sized operations (more workgroups per task) at no cost in bandwidth.
  // The same goes for a link of a chain (a task that waits for one of the few tickets right before
  // it): its successor waits for its slowest chunk, so the tail of every task is on the critical path.
  const bool chained = (t.dep[0] >= 1 && t.dep[0] <= 8) || (t.dep[1] >= 1 && t.dep[1] <= 8) || (t.dep[2] >= 1 && t.dep[2] <= 8);
  if ((numel <= (1 << 20) || chained) && chunk_elems >= 2048) chunk_elems /= 2;
  const bool red = impl_is_reduction(impl);
  const int nd_out = red ? t.ndim - 1 : t.ndim;
  Operand ops[4];                                   // inputs 0..ar-1, then the output
  for (int k = 0; k < ar; ++k) {
    const int rc = check_operand(t.in[k], t.ndim, size, false, &ops[k]);
    if (rc != GPUOS_OK) return rc;
  }
  {
    const int rc = check_operand(t.out, nd_out, size, true, &ops[ar]);
    if (rc != GPUOS_OK) return rc;
  }
  bool any_int = ops[ar].dtype == GPUOS_I32, all_int = any_int, same_dt = true;
  for (int k = 0; k < ar; ++k) {
    any_int = any_int || ops[k].dtype == GPUOS_I32;
    all_int = all_int && ops[k].dtype == GPUOS_I32;
    same_dt = same_dt && ops[k].dtype == ops[ar].dtype;
  }
  if (any_int && (!all_int || !impl_takes_int(impl))) return GPUOS_E_INVAL;
  if (all_int) rec.rflags |= RF_INT;
  rec.n_inputs = (uint8_t)ar;
  for (int k = 0; k < ar; ++k) { rec.dtype[k] = (uint8_t)ops[k].dtype; rec.ptr[k] = ops[k].ptr; }
  rec.dtype[3] = (uint8_t)ops[ar].dtype;
  rec.ptr[3] = ops[ar].ptr;

  if (impl_is_rowop(impl)) {
    // ---- fused row operation: rows of the last dim, every operand has the full rank ----
    if (numel == 0) { rec.path = PATH_NOP; rec.nchunks = 1; *r = rec; return GPUOS_OK; }
    const int64_t n = size[t.ndim - 1];
    const int64_t rows = numel / n;
    int64_t osz[GPUOS_MAX_DIMS];
    Operand oo[4];
    int64_t s_last[4];
    for (int k = 0; k <= ar; ++k) {
      oo[k] = ops[k];
      s_last[k] = n > 1 ? ops[k].stride[t.ndim - 1] : 1;
      for (int d = t.ndim - 1; d < GPUOS_MAX_DIMS; ++d) oo[k].stride[d] = 0;
    }
    for (int d = 0; d < GPUOS_MAX_DIMS; ++d) osz[d] = d < t.ndim - 1 ? size[d] : 1;
    int nd = 1;
    if (t.ndim > 1) nd = coalesce(t.ndim - 1, osz, oo, ar + 1);
    else { osz[0] = 1; for (int k = 0; k <= ar; ++k) oo[k].stride[0] = 0; }
    if (rows == 1) { nd = 1; osz[0] = 1; for (int k = 0; k <= ar; ++k) oo[k].stride[0] = 0; }
    rec.ndim = (uint8_t)nd;
    for (int k = 0; k <= ar; ++k) {
      const int kk = k < ar ? k : 3;
      for (int d = 0; d < nd; ++d) rec.stride[kk][d] = (uint32_t)oo[k].stride[d];
      rec.stride[kk][5] = (uint32_t)s_last[k];
    }
    for (int d = 0; d < nd; ++d) rec.size[d] = (uint32_t)osz[d];
    rec.red_n = (uint32_t)n;
    rec.numel = (uint32_t)rows;
    rec.path = PATH_ROW_GENERIC;
    // vector path (rows in registers up to 1024 vectors, streamed beyond): one dtype, unit stride
    // along the row, whole aligned vectors; x and the output contiguous; further inputs contiguous [period, n]
    // blocks that repeat every `period` rows (period = rows: same layout as x; 1: a row vector)
    const uint32_t es = dtype_size(ops[ar].dtype);
    const uint32_t V = 16u / es;
    auto dense_rows = [&](const Operand& o, int from) {      // dims from..nd-1 laid out as [.., n] contiguous
      int64_t want = n;
      for (int d = nd - 1; d >= from; --d) {
        if (osz[d] > 1 && o.stride[d] != want) return false;
        want *= osz[d];
      }
      return true;
    };
    // one dtype for every tensor; layer norm also with fp32 gamma and beta under 16-bit x and y
    const bool ln_p32 = impl == GPUOS_IMPL_LAYERNORM_LAST && ops[0].dtype == ops[ar].dtype && ops[0].dtype != GPUOS_F32 &&
                        ops[1].dtype == GPUOS_F32 && ops[2].dtype == GPUOS_F32;
    bool fast = (same_dt || ln_p32) && n % V == 0 && n * (int64_t)es < kMaxExtent && n * 4 < kMaxExtent;
    for (int k = 0; k <= ar && fast; ++k) fast = s_last[k] == 1 && aligned16(ops[k].ptr);
    fast = fast && (rows == 1 || (dense_rows(oo[0], 0) && dense_rows(oo[ar], 0)));
    uint32_t period[3] = {0, 0, 0};
    for (int k = 1; k < ar && fast; ++k) {
      if (rows == 1 || dense_rows(oo[k], 0)) { rec.okind[k] = K_FULL; continue; }
      int q = nd;                                            // outer dims 0..q-1 broadcast, q..nd-1 dense
      while (q > 0 && dense_rows(oo[k], q - 1) && oo[k].stride[q - 1] != 0) --q;
      // here dims q..nd-1 are dense; dims 0..q-1 must all be broadcast
      bool ok = true;
      for (int d = 0; d < q; ++d) ok = ok && (osz[d] == 1 || oo[k].stride[d] == 0);
      int64_t per = 1;
      for (int d = q; d < nd; ++d) per *= osz[d];
      if (!ok || per * n * (int64_t)es >= kMaxExtent) { fast = false; break; }
      rec.okind[k] = K_PERIODIC;
      period[k] = (uint32_t)per;
    }
    if (impl == GPUOS_IMPL_LAYERNORM_LAST && fast && rows > 1)    // gamma, beta: row vectors, loaded once per lane
      fast = rec.okind[1] == K_PERIODIC && period[1] == 1 && rec.okind[2] == K_PERIODIC && period[2] == 1;
    if (fast) {
      rec.path = PATH_ROW_FUSED;
      rec.rflags |= RF_VEC;
      for (int k = 1; k < ar; ++k) rec.stride[k][0] = period[k];
    }
    uint64_t row_bytes = 0;
    for (int k = 0; k <= ar; ++k) row_bytes += (uint64_t)n * dtype_size(ops[k].dtype);
    uint64_t rpc = (uint64_t)chunk_elems * 12 / row_bytes;
    if (rpc < 1) rpc = 1;
    if (rpc >= 16) rpc = (rpc + 15) / 16 * 16;
    const uint64_t min_rpc = ((uint64_t)rows + kMaxChunksPerTask - 1) / kMaxChunksPerTask;
    if (rpc < min_rpc) rpc = min_rpc;
    rec.chunk = (uint32_t)rpc;
    rec.nchunks = (uint32_t)(((uint64_t)rows + rpc - 1) / rpc);
    *r = rec;
    return GPUOS_OK;
  }

  if (!red) {
    if (numel == 0) { rec.path = PATH_NOP; rec.nchunks = 1; *r = rec; return GPUOS_OK; }
    const int nd = coalesce(t.ndim, size, ops, ar + 1);
    rec.ndim = (uint8_t)nd;
    for (int d = 0; d < nd; ++d) {
      rec.size[d] = (uint32_t)size[d];
      for (int k = 0; k < ar; ++k) rec.stride[k][d] = (uint32_t)ops[k].stride[d];
      rec.stride[3][d] = (uint32_t)ops[ar].stride[d];
    }
    rec.numel = (uint32_t)numel;
    const uint32_t V = 16u / dtype_size(ops[ar].dtype);
    bool all_unit = nd == 1;
    bool all_aligned = aligned16(ops[ar].ptr);
    for (int k = 0; k <= ar && all_unit; ++k) all_unit = ops[k].stride[0] == 1 || numel == 1;
    rec.path = PATH_GENERIC;
    if (all_unit && same_dt) {
      rec.path = PATH_CONTIG;
      for (int k = 0; k < ar; ++k) all_aligned = all_aligned && aligned16(ops[k].ptr);
      if (all_aligned) rec.rflags |= RF_VEC;
    } else if (!all_int && nd == 2 && ar >= 2 && ops[ar].stride[1] == 1 && ops[ar].stride[0] == size[1] &&
               size[1] % V == 0 && all_aligned && size[1] * 4 < kMaxExtent) {   // a row fits one buffer resource
      bool ok = true;
      for (int k = 0; k < ar && ok; ++k) {
        const int64_t s0 = ops[k].stride[0], s1 = ops[k].stride[1];
        if (s1 == 1 && s0 == size[1] && ops[k].dtype == ops[ar].dtype && aligned16(ops[k].ptr)) rec.okind[k] = K_FULL;
        else if (s1 == 1 && s0 == 0 && ops[k].dtype == ops[ar].dtype && aligned16(ops[k].ptr)) rec.okind[k] = K_ROWVEC;
        else if (s1 == 0) rec.okind[k] = K_ROWSCALAR;
        else ok = false;
      }
      if (ok) { rec.path = PATH_ROW2D; rec.rflags |= RF_VEC; }
    }
    // chunk_elems is quoted for 12 bytes of traffic per element (an fp32 binary op); scale it so
    // that a chunk of any op moves about the same number of bytes
    // [B, R, C] contiguous output with an input whose unit stride runs along R (a transposed
    // view): gathered through LDS tiles.  COPY between equal dtypes stays on the generic path,
    // which moves raw bits (NaN payloads survive).
    if (rec.path == PATH_GENERIC && !all_int && (nd == 2 || nd == 3) &&
        !(impl == GPUOS_IMPL_COPY && same_dt)) {
      const int o = nd - 2;                                      // index of R
      const int64_t R = size[o], C = size[o + 1], B = nd == 3 ? size[0] : 1;
      const Operand& out = ops[ar];
      bool ok = R >= 8 && C >= 8 && out.stride[o + 1] == 1 && out.stride[o] == C &&
                (nd == 2 || B == 1 || out.stride[0] == R * C);
      bool any_t = false;
      uint8_t kinds[3] = {0, 0, 0};
      for (int k = 0; k < ar && ok; ++k) {
        const int64_t sr = ops[k].stride[o], sc = ops[k].stride[o + 1];
        if (sc == 1) kinds[k] = K_FULL;
        else if (sr == 1) { kinds[k] = K_TRANSPOSED; any_t = true; }
        else ok = false;
      }
      if (ok && any_t) {
        rec.path = PATH_TILE2D;
        rec.ndim = 3;
        rec.size[0] = (uint32_t)B; rec.size[1] = (uint32_t)R; rec.size[2] = (uint32_t)C;
        for (int k = 0; k <= ar; ++k) {
          const int kk = k < ar ? k : 3;
          rec.stride[kk][0] = nd == 3 ? (uint32_t)ops[k].stride[0] : 0u;
          rec.stride[kk][1] = (uint32_t)ops[k].stride[o];
          rec.stride[kk][2] = (uint32_t)ops[k].stride[o + 1];
          if (k < ar) rec.okind[k] = kinds[k];
        }
        const uint64_t tiles = (uint64_t)B * ((R + 31) / 32) * ((C + 31) / 32);
        uint64_t per_t = (tiles + kMaxChunksPerTask - 1) / kMaxChunksPerTask;
        // tiles of 1024 elements.  A workgroup takes a tile at a time (load, transpose through LDS,
        // store: 1.5-2 us alone), so a task of few tiles is spread over as many workgroups as it
        // has tiles, up to 64, before chunks grow to the regular size.  (Two tiles per workgroup
        // at least, measured: config2 within its run-to-run spread, a lone transposed task 1.3 us
        // slower.)
        uint64_t want = chunk_elems / 1024 ? chunk_elems / 1024 : 1;
        const uint64_t spread = (tiles + 63) / 64;
        if (spread < want) want = spread;
        if (per_t < want) per_t = want;
        rec.numel = (uint32_t)tiles;
        rec.chunk = (uint32_t)per_t;
        rec.nchunks = (uint32_t)((tiles + per_t - 1) / per_t);
        *r = rec;
        return GPUOS_OK;
      }
    }
    // Contiguous output of at most three merged dims whose inputs are strided, broadcast or of another
    // dtype (stride-2 slices, row and column vectors whatever the row length, small transposes,
    // mixed precision): gathered through LDS.  COPY between equal dtypes stays on the generic path
    // (raw bits).
    if (rec.path == PATH_GENERIC && !all_int && nd <= 3 && aligned16(ops[ar].ptr) && !(impl == GPUOS_IMPL_COPY && same_dt)) {
      const Operand& out = ops[ar];
      bool out_contig = true;
      int64_t want = 1;
      for (int d = nd - 1; d >= 0; --d) {
        if (size[d] > 1 && out.stride[d] != want) out_contig = false;
        want *= size[d];
      }
      if (out_contig) {
        rec.path = PATH_STAGED;
        rec.ndim = 3;
        const int lead = 3 - nd;                                   // leading dims of size 1
        for (int d = 0; d < 3; ++d) {
          rec.size[d] = d < lead ? 1u : (uint32_t)size[d - lead];
          for (int k = 0; k < ar; ++k) rec.stride[k][d] = d < lead ? 0u : (uint32_t)ops[k].stride[d - lead];
          rec.stride[3][d] = d < lead ? 0u : (uint32_t)out.stride[d - lead];
        }
      }
    }
    uint64_t traffic = dtype_size(ops[ar].dtype);
    for (int k = 0; k < ar; ++k) traffic += dtype_size(ops[k].dtype);
    uint64_t base_per = ((uint64_t)chunk_elems * 12 / traffic + 1023) / 1024 * 1024;
    uint64_t per = ((uint64_t)numel + kMaxChunksPerTask - 1) / kMaxChunksPerTask;
    per = (per + 1023) / 1024 * 1024;
    if (per < base_per) {
      // A task of at most four regular chunks is cut into (up to) four chunks of at least half the
      // regular size.  One workgroup streams a chunk at 50-60 GB/s, so a task of 8K-32K elements that
      // runs alone (or as a link of a chain) is bound by that, not by the GPU: 16K elements take 5 us
      // in one workgroup, 3 us in four.  It stays within the four chunks up to which a dependent task
      // is published at once and waits in its workgroups.
      uint64_t quarter = (((uint64_t)numel + 3) / 4 + 1023) / 1024 * 1024;
      uint64_t half = (base_per / 2 + 1023) / 1024 * 1024;
      if (rec.path == PATH_STAGED) {
        // the gather path works in rounds of 1,024 elements (load the covering windows, stage,
        // gather, store: the first about 1.5 us, the following ones, whose loads are requested a
        // round ahead, about half of that): a task of a few dozen rounds is spread over up to 32
        // workgroups, two rounds each at least
        quarter = (((uint64_t)numel + 31) / 32 + 1023) / 1024 * 1024;
        half = 2048;
      }
      if (quarter < half) quarter = half;
      per = quarter < base_per ? quarter : base_per;
    }
    rec.chunk = (uint32_t)per;
    rec.nchunks = (uint32_t)(((uint64_t)numel + per - 1) / per);
    *r = rec;
    return GPUOS_OK;
  }

  // ---- reduction over the last dim ----
  const int64_t n = size[t.ndim - 1];
  int64_t rows = 1;
  for (int d = 0; d + 1 < t.ndim; ++d) rows *= size[d];
  if (n == 0 && rows != 0) return GPUOS_E_INVAL;    // empty reduced dim: no defined result
  if (rows == 0 || n == 0) { rec.path = PATH_NOP; rec.nchunks = 1; *r = rec; return GPUOS_OK; }
  const int64_t s_last = n > 1 ? ops[0].stride[t.ndim - 1] : 1;
  int64_t osz[GPUOS_MAX_DIMS];
  Operand oo[2] = {ops[0], ops[1]};
  for (int d = 0; d < GPUOS_MAX_DIMS; ++d) osz[d] = d < t.ndim - 1 ? size[d] : 1;
  for (int d = t.ndim - 1; d < GPUOS_MAX_DIMS; ++d) { oo[0].stride[d] = 0; oo[1].stride[d] = 0; }
  int nd = 0;
  if (t.ndim > 1) nd = coalesce(t.ndim - 1, osz, oo, 2);
  else { osz[0] = 1; oo[0].stride[0] = 0; oo[1].stride[0] = 0; nd = 1; }
  rec.ndim = (uint8_t)nd;
  for (int d = 0; d < nd; ++d) {
    rec.size[d] = (uint32_t)osz[d];
    rec.stride[0][d] = (uint32_t)oo[0].stride[d];
    rec.stride[3][d] = (uint32_t)oo[1].stride[d];
  }
  rec.stride[0][5] = (uint32_t)s_last;
  rec.red_n = (uint32_t)n;
  rec.numel = (uint32_t)rows;
  const uint32_t V = 16u / dtype_size(ops[0].dtype);
  const bool rows_contig = rows == 1 || (nd == 1 && oo[0].stride[0] == n && oo[1].stride[0] == 1);
  if (!all_int && s_last == 1 && rows_contig && n * 4 < kMaxExtent) {            // a row fits one buffer resource
    rec.path = PATH_RED_CONTIG;
    if (aligned16(ops[0].ptr)) rec.rflags |= RF_VEC;    // rows are read as aligned vectors whatever n is
  } else {
    rec.path = PATH_RED_GENERIC;
  }
  // same traffic per chunk as an elementwise chunk: chunk_elems * 12 bytes of input rows
  uint64_t rpc = (uint64_t)chunk_elems * 24 / ((uint64_t)n * dtype_size(ops[0].dtype));
  if (rpc < 1) rpc = 1;
  if (rpc >= 16) rpc = (rpc + 15) / 16 * 16;          // whole passes of the row-per-wave kernels
  const uint64_t min_rpc = ((uint64_t)rows + kMaxChunksPerTask - 1) / kMaxChunksPerTask;
  if (rpc < min_rpc) rpc = min_rpc;
  rec.chunk = (uint32_t)rpc;
  rec.nchunks = (uint32_t)(((uint64_t)rows + rpc - 1) / rpc);
  *r = rec;
  return GPUOS_OK;
}

struct OpInfo {
  uint32_t impl = 0;
  uint32_t version = 0;            // 0 = unregistered
  uint64_t prev_swap_head = 0;     // tickets submitted before the previous swap returned
};

}  // namespace

struct gpuos_ctx {
  gpuos_config cfg;
  int device = 0;
  hipStream_t stream = nullptr;
  hipEvent_t ev_start = nullptr, ev_stop = nullptr;
  uint32_t cap = 0, mask = 0, workgroups = 0;
  // host-coherent
  HostCtl* h = nullptr;
  DoorbellCtl* bell = nullptr;               // host or device memory (push mode)
  bool push = false;
  bool direct_store = false;              // push mode on a CPU with direct stores (MOVDIRI / MOVDIR64B): see direct_store_record
  Record* hring = nullptr;
  uint64_t* hcomp = nullptr;
  OpSlots* htable = nullptr;
  // device
  DevCtl* d = nullptr;
  Record* dring = nullptr;
  uint64_t* units = nullptr;
  SlotState* st = nullptr;
  OpSlots* dtable = nullptr;
  // operator programs (device-visible like the ring; written by the host)
  ProgramImage* progs = nullptr;
  uint32_t n_progs = 0;                      // changed under prod_mu
  uint8_t prog_arity[GPUOS_MAX_PROGRAMS] = {};
  // tracing (host-coherent; nullptr when off)
  TraceRec* trace = nullptr;
  uint64_t* opcount = nullptr;
  uint32_t trace_mask = 0;
  uint64_t origin_host_ns = 0;               // host clock when the worker's first heartbeat was seen
  // producer state
  SpinMutex prod_mu;                         // producers: ticket reservation, ring writes, doorbell, table changes
  std::mutex harvest_mu;                     // one harvester at a time
  std::atomic<uint64_t> head{0};             // tickets written (changed under prod_mu)
  std::atomic<uint64_t> published{0};        // tickets behind the doorbell
  std::atomic<uint64_t> floor{0};            // completed in order
  std::atomic<int32_t> first_error{0};
  uint64_t epoch = 0;
  OpInfo ops[GPUOS_MAX_OPS];
  // completion log (log points into log_store, or into the caller's block for a static context)
  std::vector<gpuos_completion> log_store;
  gpuos_completion* log = nullptr;
  uint64_t log_mask = 0;
  // harvester
  std::thread harvester;
  std::atomic<bool> harvester_run{false};
  bool worker_running = false;
  std::vector<gpuos_audit_record> audit;  // latest kAuditKeep changes of the operator table, a ring once full (under prod_mu)
  uint64_t audit_total = 0;
  bool static_mode = false;               // made by gpuos_init_static: the library owns neither the memory nor the stream
  // operator programs as native code: a second resident worker kernel compiled at run time
  ProgramImage prog_img[GPUOS_MAX_PROGRAMS] = {};   // host copy of what the device-visible table holds
  bool jit_enabled = false;               // this context may use the run-time compiler
  bool jit_failed = false;                // ... and has not given up on it
  std::mutex jit_mu;                      // one change of generation at a time (taken before prod_mu, never after)
  uint64_t* units_j = nullptr;            // the second work-unit ring
  hipStream_t jit_stream = nullptr;
  hipModule_t jit_mod = nullptr;
  hipFunction_t jit_fn = nullptr;
  uint32_t jit_gen = 0;                   // generation of the loaded module (0: none)
  uint32_t jit_n = 0;                     // programs it holds as native code
  uint32_t jit_grid = 0;
  bool jit_running = false;               // its kernel is resident
  uint64_t jit_builds = 0, jit_cache_hits = 0;
  double jit_last_ms = 0.0;
  std::string jit_error;                  // why the native path was given up (jit_failed)
  uint64_t prog_hash[GPUOS_MAX_PROGRAMS] = {};
  uint32_t prog_len[GPUOS_MAX_PROGRAMS] = {};
  WorkerArgs wargs{};                     // what the worker was launched with (gpuos_start_worker launches it again)
  bool worker_joined = false;
  uint64_t wait_ns = 0;
};

namespace {

std::mutex g_live_mu;
std::vector<gpuos_ctx*> g_live;
bool g_atexit_registered = false;

// Harvest completion words in ticket order (single consumer).
uint64_t harvest(gpuos_ctx* c) {
  std::unique_lock<std::mutex> lk(c->harvest_mu, std::try_to_lock);
  if (!lk.owns_lock()) return 0;             // another thread is harvesting: it will advance the floor
  uint64_t f = c->floor.load(std::memory_order_relaxed);
  const uint64_t pub = c->published.load(std::memory_order_acquire);
  uint64_t t_done = 0;
  uint64_t n = 0;
  while (f < pub) {
    const uint64_t w = __atomic_load_n(&c->hcomp[f & c->mask], __ATOMIC_ACQUIRE);
    if ((uint32_t)w != (uint32_t)(f + 1)) break;
    if (t_done == 0) t_done = now_ns();
    gpuos_completion& e = c->log[f & c->log_mask];
    e.ticket = f;
    e.status = (int32_t)(int8_t)(uint8_t)(w >> 32);
    e.op_version = (uint32_t)(w >> 40);
    e.t_done_ns = t_done;
    if (e.status != 0) {
      int32_t zero = 0;
      c->first_error.compare_exchange_strong(zero, e.status);
    }
    ++f;
    ++n;
  }
  if (n) c->floor.store(f, std::memory_order_release);
  return n;
}

void harvester_main(gpuos_ctx* c, int producer_cpu) {
  // pin to the last allowed core that is not the one the producer was running on when it created
  // the context: a spinning harvester on the producer's core would starve it for whole time slices
  cpu_set_t set;
  if (sched_getaffinity(0, sizeof(set), &set) == 0) {
    int pick = -1;
    for (int i = 0; i < CPU_SETSIZE; ++i) if (CPU_ISSET(i, &set) && i != producer_cpu) pick = i;
    if (pick >= 0) { cpu_set_t one; CPU_ZERO(&one); CPU_SET(pick, &one); pthread_setaffinity_np(pthread_self(), sizeof(one), &one); }
  }
  while (c->harvester_run.load(std::memory_order_acquire)) {
    if (harvest(c) == 0) __builtin_ia32_pause();
  }
  harvest(c);
}

inline bool worker_exited(gpuos_ctx* c) { return __atomic_load_n(&c->h->exit_code, __ATOMIC_ACQUIRE) != 0; }

// Spin until floor >= target.  Returns OK / TIMEOUT / DEAD.
int wait_floor(gpuos_ctx* c, uint64_t target, uint64_t timeout_ns) {
  const uint64_t t0 = now_ns();
  uint32_t spins = 0;
  while (true) {
    if (!c->harvester_run.load(std::memory_order_relaxed)) harvest(c);
    if (c->floor.load(std::memory_order_acquire) >= target) return GPUOS_OK;
    if ((++spins & 1023u) == 0) {
      if (worker_exited(c)) {
        if (!c->harvester_run.load(std::memory_order_relaxed)) harvest(c);
        return c->floor.load(std::memory_order_acquire) >= target ? GPUOS_OK : GPUOS_E_DEAD;
      }
      if (now_ns() - t0 > timeout_ns) return GPUOS_E_TIMEOUT;
    }
    __builtin_ia32_pause();
  }
}

// Direct stores (MOVDIR64B: 64 bytes as one posted write; MOVDIRI: 8 bytes) go to the device without
// sitting in a write-combining buffer, so nothing has to be flushed behind them: a lone record and its
// doorbell reach the ring without a store fence (each fence stalls the host for 0.15-0.2 us).  They are
// weakly ordered among themselves; the record's check word covers a doorbell that lands first.
bool cpu_has_direct_stores() {
  unsigned a = 0, b = 0, c = 0, d = 0;
  __asm__ volatile("cpuid" : "=a"(a), "=b"(b), "=c"(c), "=d"(d) : "a"(0), "c"(0));
  if (a < 7) return false;
  __asm__ volatile("cpuid" : "=a"(a), "=b"(b), "=c"(c), "=d"(d) : "a"(7), "c"(0));
  return ((c >> 27) & 1u) != 0 && ((c >> 28) & 1u) != 0;         // MOVDIRI, MOVDIR64B
}
__attribute__((target("movdir64b"))) void direct_store_record(Record* dst, const Record* src) {
  for (int k = 0; k < 4; ++k) _movdir64b(reinterpret_cast<char*>(dst) + 64 * k, reinterpret_cast<const char*>(src) + 64 * k);
}
__attribute__((target("movdiri"))) void direct_store_u64(uint64_t* dst, uint64_t v) {
  _directstoreu_u64(dst, v);
}

// Publish every written ticket: time-stamp, one store-release of the tail.  Caller holds prod_mu.
// fence_first = false: the caller has just written ONE record and not pushed it out of the
// write-combining buffers; record and doorbell then leave with one flush.  The doorbell may land
// first: the dispatcher reads a record that the doorbell covers until its check word holds.  (Only
// for a lone record, where the flush is a tenth of the latency: behind a batch of 64 records the
// doorbell did land first often enough to cost the small-task streams a fifth of their rate.)
void doorbell(gpuos_ctx* c, bool fence_first = true, bool direct = false) {
  const uint64_t pub = c->published.load(std::memory_order_relaxed);
  const uint64_t head = c->head.load(std::memory_order_relaxed);
  if (pub == head) return;
  const uint64_t t = now_ns();
  for (uint64_t i = pub; i < head; ++i) c->log[i & c->log_mask].t_submit_ns = t;
  c->published.store(head, std::memory_order_release);
  if (direct) {                                                 // (the lone record went out as direct stores as well)
    direct_store_u64(&c->bell->tail, head);
    return;
  }
  if (c->push && fence_first) _mm_sfence();                     // records (write-combined BAR stores) before the doorbell
  __atomic_store_n(&c->bell->tail, head, __ATOMIC_RELEASE);     // the commit: one store-release
  if (c->push) _mm_sfence();                                    // ... and push the doorbell out of the write-combining buffer
}
void doorbell_locked(gpuos_ctx* c) {
  std::lock_guard<SpinMutex> lk(c->prod_mu);
  doorbell(c);
}

void bump_epoch(gpuos_ctx* c, uint32_t op_hint, bool stop) {
  ++c->epoch;
  const uint64_t w = (c->epoch << 12) | ((uint64_t)(op_hint & 0xffu) << 4) | (stop ? 1u : 0u);
  if (c->push) _mm_sfence();
  __atomic_store_n(&c->bell->epoch_word, w, __ATOMIC_RELEASE);
  if (c->push) _mm_sfence();
}

void free_all(gpuos_ctx* c) {
  if (c->static_mode) return;               // the caller's host block and stream, the library's device array: nothing to free
  if (c->jit_mod) (void)hipModuleUnload(c->jit_mod);
  if (c->units_j) (void)hipFree(c->units_j);
  if (c->jit_stream) (void)hipStreamDestroy(c->jit_stream);
  c->jit_mod = nullptr; c->jit_fn = nullptr; c->units_j = nullptr; c->jit_stream = nullptr;
  if (c->h) (void)hipHostFree(c->h);
  if (c->hcomp) (void)hipHostFree(c->hcomp);
  if (c->trace) (void)hipHostFree(c->trace);
  if (c->opcount) (void)hipHostFree(c->opcount);
  c->trace = nullptr; c->opcount = nullptr;
  if (c->push) {
    if (c->progs) (void)hipFree(c->progs);
    if (c->bell) (void)hipFree(c->bell);
    if (c->hring) (void)hipFree(c->hring);
    if (c->htable) (void)hipFree(c->htable);
  } else {
    if (c->progs) (void)hipHostFree(c->progs);
    if (c->bell) (void)hipHostFree(c->bell);
    if (c->hring) (void)hipHostFree(c->hring);
    if (c->htable) (void)hipHostFree(c->htable);
  }
  if (c->d) (void)hipFree(c->d);
  if (c->dring) (void)hipFree(c->dring);
  if (c->units) (void)hipFree(c->units);
  if (c->st) (void)hipFree(c->st);
  if (c->dtable) (void)hipFree(c->dtable);
  if (c->ev_start) (void)hipEventDestroy(c->ev_start);
  if (c->ev_stop) (void)hipEventDestroy(c->ev_stop);
  if (c->stream) (void)hipStreamDestroy(c->stream);
  c->progs = nullptr;
  c->h = nullptr; c->bell = nullptr; c->hring = nullptr; c->hcomp = nullptr; c->htable = nullptr;
  c->d = nullptr; c->dring = nullptr; c->units = nullptr; c->st = nullptr; c->dtable = nullptr;
  c->ev_start = nullptr; c->ev_stop = nullptr; c->stream = nullptr;
}

// Mark programs [0, jit_n) as served natively (v = 1) or interpreted (v = 0) in the device-visible
// table; with `announce` the dispatcher is told to read the flags again.  Caller holds jit_mu or is the
// only thread (stop / start).
void jit_set_native(gpuos_ctx* c, uint32_t v, bool announce) {
  std::lock_guard<SpinMutex> lk(c->prod_mu);
  for (uint32_t k = 0; k < c->jit_n && k < GPUOS_MAX_PROGRAMS; ++k) {
    c->prog_img[k].native = v;
    __atomic_store_n(&c->progs[k].native, v, __ATOMIC_RELAXED);
  }
  if (c->push) _mm_sfence();
  if (announce) bump_epoch(c, 0xff, false);
}

int stop_worker(gpuos_ctx* c) {
  if (c->worker_joined) return GPUOS_OK;
  int rc = GPUOS_OK;
  if (c->worker_running) {
    if (!worker_exited(c)) {                                  // (one that left by itself is only joined)
      doorbell_locked(c);
      rc = wait_floor(c, c->head.load(), c->wait_ns);         // drain
    }
    {
      std::lock_guard<SpinMutex> lk(c->prod_mu);              // the epoch is the producers' (a swap may be running)
      bump_epoch(c, 0xff, true);                              // signal worker exit
    }
    const uint64_t t0 = now_ns();
    hipError_t q;
    while ((q = hipStreamQuery(c->stream)) == hipErrorNotReady) {
      const uint64_t waited = now_ns() - t0;
      if (waited > c->wait_ns) break;
      // the kernel leaves within tens of microseconds of the flag: poll tightly at first (a caller
      // that hands the GPU to another kernel waits for exactly this), back off afterwards
      if (waited > 300000ull) std::this_thread::sleep_for(std::chrono::microseconds(50));
    }
    if (q == hipErrorNotReady) rc = GPUOS_E_TIMEOUT;
    else if (q != hipSuccess) { hip_ok(q, "worker kernel"); rc = GPUOS_E_HIP; }
    bool jit_left = true;
    if (c->jit_running) {                                     // the run-time kernel's workers obey the same stop flag
      hipError_t qj;
      while ((qj = hipStreamQuery(c->jit_stream)) == hipErrorNotReady && now_ns() - t0 <= c->wait_ns)
        std::this_thread::sleep_for(std::chrono::microseconds(20));
      jit_left = qj != hipErrorNotReady;
      if (!jit_left) rc = GPUOS_E_TIMEOUT;
      else if (qj != hipSuccess && rc == GPUOS_OK) { hip_ok(qj, "run-time worker kernel"); rc = GPUOS_E_HIP; }
      if (jit_left) {
        c->jit_running = false;
        jit_set_native(c, 0, false);                          // a restarted worker interprets until the run-time kernel is back
      }
    }
    c->worker_running = false;
    c->worker_joined = q != hipErrorNotReady && jit_left;     // the kernels have left the GPU (whatever the drain said)
  } else if (c->stream) {
    // an earlier stop ran into its time limit with a kernel still resident: look again
    if (hipStreamQuery(c->stream) == hipErrorNotReady || (c->jit_running && hipStreamQuery(c->jit_stream) == hipErrorNotReady))
      rc = GPUOS_E_TIMEOUT;
    else { c->worker_joined = true; c->jit_running = false; }
  }
  if (c->harvester_run.load()) {
    c->harvester_run.store(false, std::memory_order_release);
    if (c->harvester.joinable()) c->harvester.join();
  }
  if (c->worker_joined) harvest(c);
  return rc;
}

constexpr int kMaxStaticDevices = 64;
std::atomic<gpuos_ctx*> g_static_owner[kMaxStaticDevices];       // the context that holds a device's static array

void shutdown_all_at_exit() {
  std::vector<gpuos_ctx*> live;
  {
    std::lock_guard<std::mutex> lk(g_live_mu);
    live = g_live;
  }
  for (gpuos_ctx* c : live) (void)stop_worker(c);
  for (auto& o : g_static_owner)
    if (gpuos_ctx* c = o.load()) (void)stop_worker(c);
}

}  // namespace


namespace {
// Size the grid, launch the persistent worker for the first time and wait for its first heartbeat.
// On GPUOS_E_TIMEOUT with !worker_joined the kernel is still queued: the caller must keep the memory.
int launch_first_worker(gpuos_ctx* c, int compute_units, size_t n_units) {
  const gpuos_config& cfg = c->cfg;
  // size the grid to what is co-resident: every workgroup must be running for
  // the spin-waits (claims, dependencies) to be deadlock-free
  int occ = 0;
  if (!hip_ok((hipError_t)worker_max_blocks_per_cu(&occ), "hipOccupancyMaxActiveBlocksPerMultiprocessor")) return GPUOS_E_HIP;
  if (occ < 1) return GPUOS_E_HIP;
  uint32_t per_cu = cfg.workgroups_per_cu;
  if (per_cu > (uint32_t)occ) per_cu = (uint32_t)occ;
  c->workgroups = (uint32_t)compute_units * per_cu;
  if (c->workgroups < 2) c->workgroups = 2;
  c->cfg.workgroups_per_cu = per_cu;
  if (c->jit_enabled) {
    // The run-time kernel is built like the worker (same registers per lane, slightly less local
    // memory): its workgroups take places per compute unit that the worker leaves free.  Unless the
    // caller names their number, one place per compute unit stays free for everybody else's kernels
    // (the HIP runtime's copy kernels included: with every register file full they start only when a
    // worker leaves); with the default three workgroups per compute unit of the worker itself that
    // leaves none for the run-time kernel, and programs are interpreted.
    uint32_t jw = cfg.jit_workgroups_per_cu;
    if (jw == 0) jw = (uint32_t)occ > per_cu + 1u ? 1u : 0u;
    else if (per_cu + jw > (uint32_t)occ) jw = (uint32_t)occ > per_cu ? (uint32_t)occ - per_cu : 0u;
    c->cfg.jit_workgroups_per_cu = jw;
    c->jit_grid = (uint32_t)compute_units * jw;
    if (jw == 0) {
      c->jit_enabled = false;
      c->jit_error = "no place beside the worker's workgroups that leaves one per compute unit free: lower cfg.workgroups_per_cu, "
                     "or name cfg.jit_workgroups_per_cu to fill the compute units";
    }
  }

  WorkerArgs a{};
  a.h = c->h; a.bell = c->bell; a.hring = c->hring; a.hcomp = c->hcomp; a.htable = c->htable;
  a.d = c->d; a.dring = c->dring; a.units = c->units; a.st = c->st; a.dtable = c->dtable;
  a.units_j = c->jit_enabled ? c->units_j : nullptr;
  a.cap_mask = c->mask;
  a.unit_mask = (uint32_t)(n_units - 1);
  a.unit_shift = 0;
  while (((size_t)1 << a.unit_shift) < n_units) ++a.unit_shift;
  a.cap_shift = 0;
  while ((1u << a.cap_shift) < c->cap) ++a.cap_shift;
  a.idle_exit_ticks = (uint64_t)cfg.idle_exit_ms * 100000ull;     // 100 MHz counter
  a.progs = c->progs;
  a.trace = c->trace; a.opcount = c->opcount; a.trace_mask = c->trace_mask;
  a.resume = 0; a.resume_tickets = 0;
  a.timing = cfg.phase_timers ? 1u : 0u;
  a.dep_wait_ticks = cfg.dep_wait_us ? (uint64_t)cfg.dep_wait_us * 100ull : (uint64_t)cfg.wait_timeout_ms * 100000ull;
  c->wargs = a;
  if (c->ev_start && !hip_ok(hipEventRecord(c->ev_start, c->stream), "hipEventRecord")) return GPUOS_E_HIP;
  if (!hip_ok((hipError_t)launch_worker(a, c->workgroups, c->stream), "launch worker")) return GPUOS_E_HIP;
  if (c->ev_stop && !hip_ok(hipEventRecord(c->ev_stop, c->stream), "hipEventRecord")) return GPUOS_E_HIP;
  c->worker_running = true;

  // wait for the first heartbeat so that init returns with a live worker
  {
    const uint64_t t0 = now_ns();
    uint32_t spins = 0;
    while (__atomic_load_n(&c->h->heartbeat, __ATOMIC_ACQUIRE) == 0) {
      if ((spins & 255u) == 0 && now_ns() - t0 > c->wait_ns) {
        // The kernel never started (the device is busy with other work).  Ask it to exit as soon as it
        // does; if it still has not finished, its memory must stay: freeing under a queued
        // kernel would fault when it finally runs.
        (void)stop_worker(c);
        return GPUOS_E_TIMEOUT;
      }
      // look at the stream only now and then: the moment the heartbeat is seen ties the device
      // clock to the host clock, and a stream query takes microseconds
      if ((++spins & 4095u) == 0 && hipStreamQuery(c->stream) != hipErrorNotReady) return GPUOS_E_DEAD;
      __builtin_ia32_pause();
    }
  }
  c->origin_host_ns = now_ns();
  if (cfg.harvester_thread) {
    c->harvester_run.store(true);
    c->harvester = std::thread(harvester_main, c, sched_getcpu());
  }
  if (!c->static_mode) {
    std::lock_guard<std::mutex> lk(g_live_mu);
    g_live.push_back(c);
  }
  {
    std::lock_guard<std::mutex> lk(g_live_mu);
    if (!g_atexit_registered) { std::atexit(shutdown_all_at_exit); g_atexit_registered = true; }
  }
  return GPUOS_OK;
}
}  // namespace

extern "C" {

void gpuos_default_config(gpuos_config* cfg) {
  if (!cfg) return;
  std::memset(cfg, 0, sizeof(*cfg));
  int dev = 0;
  (void)hipGetDevice(&dev);
  cfg->device = dev;
  cfg->threads_per_workgroup = kThreads;
  cfg->workgroups_per_cu = 3;
  cfg->wait_timeout_ms = 30000;
  cfg->completion_log = 1u << 20;
  cfg->chunk_elems = kChunkElems;
  cfg->push_ring = 2;               // device-memory ring when the BAR allows it
  cfg->jit_workgroups_per_cu = 0;      // as many as leave a place per compute unit free (see launch_first_worker)
}

int gpuos_init(gpuos_ctx** out, uint32_t queue_capacity, const gpuos_config* user_cfg) {
  if (!out) return GPUOS_E_INVAL;
  *out = nullptr;
  gpuos_config cfg;
  if (user_cfg) cfg = *user_cfg; else gpuos_default_config(&cfg);
  if (cfg.threads_per_workgroup == 0) cfg.threads_per_workgroup = kThreads;
  if (cfg.threads_per_workgroup != kThreads) return GPUOS_E_INVAL;
  if (cfg.workgroups_per_cu == 0) cfg.workgroups_per_cu = 3;
  if (cfg.wait_timeout_ms == 0) cfg.wait_timeout_ms = 30000;
  if (cfg.completion_log == 0) cfg.completion_log = 1u << 20;
  if (cfg.chunk_elems == 0) cfg.chunk_elems = kChunkElems;
  cfg.chunk_elems = (cfg.chunk_elems + 1023u) / 1024u * 1024u;
  uint32_t cap = queue_capacity ? queue_capacity : 4096u;
  if (cap < 2 || cap > 65536 || (cap & (cap - 1)) != 0) return GPUOS_E_INVAL;
  const char* env_jit = std::getenv("GPUOS_JIT");                 // GPUOS_JIT=0: operator programs stay interpreted
  if (env_jit && env_jit[0] == '0') cfg.jit_mode = 2;
  const char* env_idle = std::getenv("GPUOS_IDLE_EXIT_MS");
  if (env_idle && cfg.idle_exit_ms == 0) cfg.idle_exit_ms = (uint32_t)std::strtoul(env_idle, nullptr, 10);

  gpuos_ctx* c = new (std::nothrow) gpuos_ctx();
  if (!c) return GPUOS_E_NOMEM;
  c->cfg = cfg;
  c->device = cfg.device;
  c->cap = cap;
  c->mask = cap - 1;
  c->wait_ns = (uint64_t)cfg.wait_timeout_ms * 1000000ull;
  uint64_t logcap = 1;
  while (logcap < cfg.completion_log || logcap < cap) logcap <<= 1;
  try {
    c->log_store.assign(logcap, gpuos_completion{});
  } catch (const std::bad_alloc&) {                             // no exception may cross the C boundary
    delete c;
    return GPUOS_E_NOMEM;
  }
  c->log = c->log_store.data();
  c->log_mask = logcap - 1;

  auto fail = [&](int rc) { free_all(c); delete c; return rc; };
  if (!hip_ok(hipSetDevice(cfg.device), "hipSetDevice")) return fail(GPUOS_E_HIP);
  hipDeviceProp_t prop;
  if (!hip_ok(hipGetDeviceProperties(&prop, cfg.device), "hipGetDeviceProperties")) return fail(GPUOS_E_HIP);
  const unsigned hflags = hipHostMallocCoherent | hipHostMallocMapped;
  const size_t n_units = (size_t)cap * kMaxChunksPerTask;
  c->push = cfg.push_ring == 1;
  if (cfg.push_ring >= 2) {
    int large_bar = 0;
    if (hipDeviceGetAttribute(&large_bar, hipDeviceAttributeIsLargeBar, cfg.device) != hipSuccess) large_bar = 0;
    c->push = large_bar != 0;
  }
  c->cfg.push_ring = c->push ? 1u : 0u;
  const char* env_ds = std::getenv("GPUOS_DIRECT_STORES");
  c->direct_store = c->push && cpu_has_direct_stores() && !(env_ds && env_ds[0] == '0');
  auto to_device_alloc = [&](void** p, size_t n, const char* what) {
    // memory the host writes and the device reads: pinned host memory, or (push mode) device
    // memory that the host reaches through the BAR
    return c->push ? hip_ok(hipMalloc(p, n), what) : hip_ok(hipHostMalloc(p, n, hflags), what);
  };
  if (!hip_ok(hipHostMalloc((void**)&c->h, sizeof(HostCtl), hflags), "hipHostMalloc(ctl)") ||
      !to_device_alloc((void**)&c->bell, sizeof(DoorbellCtl), "alloc(doorbell)") ||
      !to_device_alloc((void**)&c->hring, sizeof(Record) * cap, "alloc(ring)") ||
      !hip_ok(hipHostMalloc((void**)&c->hcomp, sizeof(uint64_t) * cap, hflags), "hipHostMalloc(comp)") ||
      !to_device_alloc((void**)&c->htable, sizeof(OpSlots) * GPUOS_MAX_OPS, "alloc(table)") ||
      !to_device_alloc((void**)&c->progs, sizeof(ProgramImage) * GPUOS_MAX_PROGRAMS, "alloc(programs)") ||
      !hip_ok(hipMalloc((void**)&c->d, sizeof(DevCtl)), "hipMalloc(ctl)") ||
      !hip_ok(hipMalloc((void**)&c->dring, sizeof(Record) * cap), "hipMalloc(ring)") ||
      !hip_ok(hipMalloc((void**)&c->units, sizeof(uint64_t) * n_units), "hipMalloc(units)") ||
      !hip_ok(hipMalloc((void**)&c->st, sizeof(SlotState) * cap), "hipMalloc(slots)") ||
      !hip_ok(hipMalloc((void**)&c->dtable, sizeof(OpSlots) * GPUOS_MAX_OPS), "hipMalloc(table)"))
    return fail(GPUOS_E_HIP);
  // operator programs as native code: on unless switched off or the run-time compiler is not there
  c->jit_enabled = cfg.jit_mode != 2 && jit_compiler_available();
  if (!c->jit_enabled) c->jit_error = cfg.jit_mode == 2 ? "switched off (cfg.jit_mode)" : "the HIP run-time compiler library was not found";
  if (c->jit_enabled &&
      (!hip_ok(hipMalloc((void**)&c->units_j, sizeof(uint64_t) * n_units), "hipMalloc(second unit ring)") ||
       !hip_ok(hipStreamCreateWithFlags(&c->jit_stream, hipStreamNonBlocking), "hipStreamCreateWithFlags")))
    return fail(GPUOS_E_HIP);
  std::memset(c->h, 0, sizeof(HostCtl));
  std::memset(c->hcomp, 0, sizeof(uint64_t) * cap);
  if (cfg.trace_entries) {
    uint32_t te = 1;
    while (te < cfg.trace_entries && te < (1u << 20)) te <<= 1;
    if (te < cap) te = cap;                                   // every in-flight ticket has an entry of its own
    if (!hip_ok(hipHostMalloc((void**)&c->trace, sizeof(TraceRec) * te, hflags), "hipHostMalloc(trace)") ||
        !hip_ok(hipHostMalloc((void**)&c->opcount, sizeof(uint64_t) * GPUOS_MAX_OPS, hflags), "hipHostMalloc(opcount)"))
      return fail(GPUOS_E_HIP);
    std::memset(c->trace, 0xff, sizeof(TraceRec) * te);       // ticket = ~0: no record yet
    std::memset(c->opcount, 0, sizeof(uint64_t) * GPUOS_MAX_OPS);
    c->trace_mask = te - 1;
    c->cfg.trace_entries = te;
  }
  if (c->push) {
    if (!hip_ok(hipMemset(c->bell, 0, sizeof(DoorbellCtl)), "hipMemset") ||
        !hip_ok(hipMemset(c->hring, 0, sizeof(Record) * cap), "hipMemset") ||
        !hip_ok(hipMemset(c->htable, 0, sizeof(OpSlots) * GPUOS_MAX_OPS), "hipMemset") ||
        !hip_ok(hipMemset(c->progs, 0, sizeof(ProgramImage) * GPUOS_MAX_PROGRAMS), "hipMemset"))
      return fail(GPUOS_E_HIP);
  } else {
    std::memset(c->bell, 0, sizeof(DoorbellCtl));
    std::memset(c->hring, 0, sizeof(Record) * cap);
    std::memset(c->htable, 0, sizeof(OpSlots) * GPUOS_MAX_OPS);
    std::memset(c->progs, 0, sizeof(ProgramImage) * GPUOS_MAX_PROGRAMS);
  }
  if (!hip_ok(hipStreamCreateWithFlags(&c->stream, hipStreamNonBlocking), "hipStreamCreateWithFlags") ||
      !hip_ok(hipEventCreate(&c->ev_start), "hipEventCreate") ||
      !hip_ok(hipEventCreate(&c->ev_stop), "hipEventCreate") ||
      !hip_ok(hipMemsetAsync(c->d, 0, sizeof(DevCtl), c->stream), "hipMemsetAsync") ||
      !hip_ok(hipMemsetAsync(c->st, 0, sizeof(SlotState) * cap, c->stream), "hipMemsetAsync") ||
      !hip_ok(hipMemsetAsync(c->units, 0, sizeof(uint64_t) * n_units, c->stream), "hipMemsetAsync") ||
      // The mirror ring too: a worker takes a mirrored record on the strength of its check word and
      // ticket alone, and the allocator hands a new context the block an earlier context of this
      // process freed, where the record of that context's task with the same ticket would pass.
      !hip_ok(hipMemsetAsync(c->dring, 0, sizeof(Record) * cap, c->stream), "hipMemsetAsync") ||
      !hip_ok(hipMemsetAsync(c->dtable, 0, sizeof(OpSlots) * GPUOS_MAX_OPS, c->stream), "hipMemsetAsync") ||
      (c->units_j && !hip_ok(hipMemsetAsync(c->units_j, 0, sizeof(uint64_t) * n_units, c->stream), "hipMemsetAsync")) ||
      !hip_ok(hipStreamSynchronize(c->stream), "hipStreamSynchronize"))
    return fail(GPUOS_E_HIP);

  {
    const int rc = launch_first_worker(c, prop.multiProcessorCount, n_units);
    if (rc == GPUOS_E_TIMEOUT && !c->worker_joined) return rc;    // the kernel may still start: its memory stays
    if (rc != GPUOS_OK) return fail(rc);
  }
  marker(cfg.markers != 0, "gpuos: worker launched, %llu workgroups, ring of %llu slots", c->workgroups, c->cap);
  *out = c;
  return GPUOS_OK;
}

namespace {
// Where the host-side pieces of a static context lie inside the caller's block.
struct StaticHostLayout { size_t ctx, h, bell, ring, comp, table, progs, log, total; };
constexpr StaticHostLayout static_host_layout(uint32_t cap) {
  StaticHostLayout l{};
  l.ctx = 0;
  l.h = align_up(l.ctx + sizeof(gpuos_ctx), 256);
  l.bell = align_up(l.h + sizeof(HostCtl), 256);
  l.ring = align_up(l.bell + sizeof(DoorbellCtl), 256);
  l.comp = align_up(l.ring + sizeof(Record) * cap, 256);
  l.table = align_up(l.comp + sizeof(uint64_t) * cap, 256);
  l.progs = align_up(l.table + sizeof(OpSlots) * GPUOS_MAX_OPS, 256);
  l.log = align_up(l.progs + sizeof(ProgramImage) * GPUOS_MAX_PROGRAMS, 256);
  l.total = align_up(l.log + sizeof(gpuos_completion) * cap, 256);
  return l;
}
static_assert(static_host_layout(GPUOS_STATIC_MAX_CAPACITY).total <= GPUOS_STATIC_HOST_BYTES(GPUOS_STATIC_MAX_CAPACITY) &&
              static_host_layout(2).total <= GPUOS_STATIC_HOST_BYTES(2), "GPUOS_STATIC_HOST_BYTES must cover the layout");
static_assert(GPUOS_STATIC_MAX_CAPACITY == kStaticMaxCapacity, "one limit");
}  // namespace

int gpuos_init_static(gpuos_ctx** out, uint32_t queue_capacity, const gpuos_config* user_cfg,
                      void* host_block, uint64_t host_bytes, void* stream) {
  if (!out) return GPUOS_E_INVAL;
  *out = nullptr;
  gpuos_config cfg;
  if (user_cfg) cfg = *user_cfg; else gpuos_default_config(&cfg);
  if (cfg.threads_per_workgroup == 0) cfg.threads_per_workgroup = kThreads;
  if (cfg.workgroups_per_cu == 0) cfg.workgroups_per_cu = 3;
  if (cfg.wait_timeout_ms == 0) cfg.wait_timeout_ms = 30000;
  if (cfg.chunk_elems == 0) cfg.chunk_elems = kChunkElems;
  cfg.chunk_elems = (cfg.chunk_elems + 1023u) / 1024u * 1024u;
  const uint32_t cap = queue_capacity ? queue_capacity : kStaticMaxCapacity;
  auto reject = [](const char* why) { g_hip_error = std::string("gpuos_init_static: ") + why; return GPUOS_E_INVAL; };
  if (cfg.threads_per_workgroup != kThreads) return reject("only 256 threads per workgroup are built");
  if (cap < 2 || (cap & (cap - 1)) != 0) return reject("queue_capacity must be a power of two >= 2");
  if (cap > kStaticMaxCapacity) return reject("queue_capacity exceeds GPUOS_STATIC_MAX_CAPACITY (1024): the device-side state would not fit the static array");
  if (cfg.device < 0 || cfg.device >= kMaxStaticDevices) return reject("device ordinal out of range");
  if (cfg.harvester_thread || cfg.trace_entries) return reject("harvester_thread and trace_entries need allocations: not available here");
  if (!host_block || ((uintptr_t)host_block & 255u) != 0) return reject("host_block must be 256-byte aligned");
  const StaticHostLayout hl = static_host_layout(cap);
  if (host_bytes < hl.total) return reject("host_block is smaller than GPUOS_STATIC_HOST_BYTES(queue_capacity)");
  if (!stream) return reject("a stream of the caller's is required (not the null stream)");

  // One static context per device: the array is shared by every call on that GPU.
  gpuos_ctx* expected = nullptr;
  gpuos_ctx* const self = reinterpret_cast<gpuos_ctx*>((char*)host_block + hl.ctx);
  if (!g_static_owner[cfg.device].compare_exchange_strong(expected, self)) {
    g_hip_error = "gpuos_init_static: this device's static array is held by a live context";
    return GPUOS_E_FULL;
  }
  auto release = [&](int rc) { g_static_owner[cfg.device].store(nullptr); return rc; };
  if (!hip_ok(hipSetDevice(cfg.device), "hipSetDevice")) return release(GPUOS_E_HIP);
  int cus = 0;
  if (!hip_ok(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, cfg.device), "hipDeviceGetAttribute") || cus < 1)
    return release(GPUOS_E_HIP);
  void* base = nullptr;                                          // this device's copy of the static array
  if (!hip_ok((hipError_t)static_scratch(cfg.device, &base), "hipGetSymbolAddress(scratch)")) return release(GPUOS_E_HIP);

  std::memset(host_block, 0, hl.total);
  gpuos_ctx* c = new (self) gpuos_ctx();                         // placement: no allocation
  c->static_mode = true;
  cfg.push_ring = 0;                                             // the ring lives in the caller's host memory
  cfg.completion_log = cap;
  c->cfg = cfg;
  c->device = cfg.device;
  c->cap = cap;
  c->mask = cap - 1;
  c->wait_ns = (uint64_t)cfg.wait_timeout_ms * 1000000ull;
  char* hb = (char*)host_block;
  c->h = (HostCtl*)(hb + hl.h);
  c->bell = (DoorbellCtl*)(hb + hl.bell);
  c->hring = (Record*)(hb + hl.ring);
  c->hcomp = (uint64_t*)(hb + hl.comp);
  c->htable = (OpSlots*)(hb + hl.table);
  c->progs = (ProgramImage*)(hb + hl.progs);
  c->log = (gpuos_completion*)(hb + hl.log);
  c->log_mask = cap - 1;
  c->push = false;
  c->stream = (hipStream_t)stream;
  const StaticLayout dl = static_layout(cap);
  char* db = (char*)base;
  c->d = (DevCtl*)(db + dl.d);
  c->dring = (Record*)(db + dl.dring);
  c->units = (uint64_t*)(db + dl.units);
  c->st = (SlotState*)(db + dl.st);
  c->dtable = (OpSlots*)(db + dl.dtable);
  const size_t n_units = (size_t)cap * kMaxChunksPerTask;
  auto fail = [&](int rc) { c->~gpuos_ctx(); return release(rc); };
  // The array keeps what the previous context left in it: everything this one reads before it
  // writes starts at zero (counters, stamps of the unit ring, done words, the table).  Same
  // stream as the worker, so the kernel starts after the clears.
  if (!hip_ok(hipMemsetAsync(base, 0, dl.total, c->stream), "hipMemsetAsync(scratch)")) return fail(GPUOS_E_HIP);
  const int rc = launch_first_worker(c, cus, n_units);
  if (rc == GPUOS_E_TIMEOUT && !c->worker_joined) return rc;      // the kernel may still start: the array stays taken
  if (rc != GPUOS_OK) return fail(rc);
  *out = c;
  return GPUOS_OK;
}

namespace {
constexpr size_t kAuditKeep = 65536;
// caller holds prod_mu
void audit(gpuos_ctx* c, uint32_t kind, uint32_t op_id, uint32_t impl_id, uint32_t version) {
  gpuos_audit_record r{};
  r.t_ns = now_ns();
  r.head_ticket = c->head.load(std::memory_order_relaxed);
  r.kind = kind; r.op_id = op_id; r.impl_id = impl_id; r.version = version;
  if (impl_id >= GPUOS_IMPL_PROGRAM_BASE && impl_id - GPUOS_IMPL_PROGRAM_BASE < GPUOS_MAX_PROGRAMS) {
    const uint32_t k = impl_id - GPUOS_IMPL_PROGRAM_BASE;
    r.n_instr = c->prog_len[k]; r.n_inputs = c->prog_arity[k]; r.code_hash = c->prog_hash[k];
  }
  static const char* const what[5] = {"", "register", "swap", "kill", "define program"};
  if (c->cfg.markers) {
    char buf[96];
    std::snprintf(buf, sizeof(buf), "gpuos %s: op %u impl %u version %u from ticket %llu", what[kind], op_id, impl_id, version,
                  (unsigned long long)r.head_ticket);
    if (roctx().mark) roctx().mark(buf);
  }
  if (c->audit.size() < kAuditKeep) c->audit.push_back(r);
  else c->audit[(size_t)(c->audit_total % kAuditKeep)] = r;
  ++c->audit_total;
}
// built-in implementation, or a program this context has defined (caller holds prod_mu)
bool impl_known(const gpuos_ctx* c, uint32_t impl) {
  if (impl != GPUOS_IMPL_NONE && impl < GPUOS_IMPL_COUNT) return true;
  return impl >= GPUOS_IMPL_PROGRAM_BASE && impl - GPUOS_IMPL_PROGRAM_BASE < c->n_progs;
}
int ctx_impl_arity(const gpuos_ctx* c, uint32_t impl) {
  return impl >= GPUOS_IMPL_PROGRAM_BASE ? (int)c->prog_arity[impl - GPUOS_IMPL_PROGRAM_BASE] : impl_arity(impl);
}
}  // namespace

namespace {

void jit_give_up(gpuos_ctx* c, const std::string& why) {
  c->jit_failed = true;
  c->jit_error = why;
  jit_set_native(c, 0, c->worker_running && !worker_exited(c));      // everything is interpreted from here on
}

// Launch the loaded module's kernel (generation c->jit_gen) and wait until its first workgroup runs.
int jit_launch(gpuos_ctx* c) {
  WorkerArgs a = c->wargs;
  uint32_t gen = c->jit_gen;
  void* params[2] = {&a, &gen};
  __atomic_store_n(&c->h->jit_alive, 0u, __ATOMIC_RELEASE);
  // after whatever the worker's stream did before the worker started (the fix-up of a restart)
  if (c->ev_start) HIP_TRY(hipStreamWaitEvent(c->jit_stream, c->ev_start, 0));
  HIP_TRY(hipModuleLaunchKernel(c->jit_fn, c->jit_grid, 1, 1, kThreads, 1, 1, 0, c->jit_stream, params, nullptr));
  c->jit_running = true;
  const uint64_t t0 = now_ns();
  const uint64_t limit = c->wait_ns < 5000000000ull ? c->wait_ns : 5000000000ull;
  while (__atomic_load_n(&c->h->jit_alive, __ATOMIC_ACQUIRE) != gen) {
    if (now_ns() - t0 > limit) return GPUOS_E_TIMEOUT;               // no compute unit had room for it
    if (hipStreamQuery(c->jit_stream) != hipErrorNotReady) { c->jit_running = false; return GPUOS_E_DEAD; }
    __builtin_ia32_pause();
  }
  return GPUOS_OK;
}

// Make the running kernel of generation c->jit_gen leave while the worker runs on: take its programs
// off the second ring, wait until everything that may have been routed there has completed, ask for
// the next generation, join.  Caller holds jit_mu.
int jit_retire(gpuos_ctx* c) {
  uint64_t head0;
  {
    jit_set_native(c, 0, true);
    std::lock_guard<SpinMutex> lk(c->prod_mu);
    head0 = c->head.load(std::memory_order_relaxed);
    doorbell(c);
  }
  // tickets from head0 on were published after the flags went down and are interpreted; earlier ones
  // may sit on the second ring
  const int rc = wait_floor(c, head0, c->wait_ns);
  if (rc != GPUOS_OK) return rc;
  {
    std::lock_guard<SpinMutex> lk(c->prod_mu);
    __atomic_store_n(&c->bell->jit_gen, c->jit_gen + 1, __ATOMIC_RELEASE);
    bump_epoch(c, 0xff, false);
  }
  const uint64_t t0 = now_ns();
  hipError_t q;
  while ((q = hipStreamQuery(c->jit_stream)) == hipErrorNotReady) {
    if (now_ns() - t0 > c->wait_ns) return GPUOS_E_TIMEOUT;
    std::this_thread::sleep_for(std::chrono::microseconds(20));
  }
  c->jit_running = false;
  if (q != hipSuccess) { hip_ok(q, "run-time worker kernel"); return GPUOS_E_HIP; }
  return GPUOS_OK;
}

// Bring the native code up to date with the programs defined so far: compile (or take from the
// cache) a worker kernel that holds all of them, retire the one that is running, launch the new one,
// route the programs' tasks to it.  Failures are not errors of the caller's: the programs stay
// interpreted.
void jit_install(gpuos_ctx* c) {
  std::lock_guard<std::mutex> jl(c->jit_mu);
  if (!c->jit_enabled || c->jit_failed) return;
  uint32_t n;
  std::vector<ProgramImage> imgs;
  {
    std::lock_guard<SpinMutex> lk(c->prod_mu);
    n = c->n_progs;
    imgs.assign(c->prog_img, c->prog_img + n);
  }
  if (n == 0 || (c->jit_mod && n == c->jit_n)) return;
  std::vector<char> code;
  std::string err;
  bool hit = false;
  double ms = 0.0;
  if (jit_build(imgs.data(), n, &code, &err, &ms, &hit) != 0) { jit_give_up(c, err); return; }
  if (hit) ++c->jit_cache_hits; else { ++c->jit_builds; c->jit_last_ms = ms; }
  if (hipSetDevice(c->device) != hipSuccess) { jit_give_up(c, "hipSetDevice"); return; }
  const bool live = c->worker_running && !worker_exited(c);
  if (c->jit_running) {
    if (!live) { jit_give_up(c, "the worker left while its run-time kernel was resident"); return; }
    const int rc = jit_retire(c);
    if (rc != GPUOS_OK) { jit_give_up(c, std::string("retiring the previous run-time kernel: ") + gpuos_strerror(rc)); return; }
  }
  if (c->jit_mod) { (void)hipModuleUnload(c->jit_mod); c->jit_mod = nullptr; c->jit_fn = nullptr; }
  hipModule_t mod = nullptr;
  hipFunction_t fn = nullptr;
  if (hipModuleLoadData(&mod, code.data()) != hipSuccess || hipModuleGetFunction(&fn, mod, "gpuos_native_worker") != hipSuccess) {
    if (mod) (void)hipModuleUnload(mod);
    jit_give_up(c, "loading the compiled worker kernel failed");
    return;
  }
  c->jit_mod = mod;
  c->jit_fn = fn;
  c->jit_gen += 1;
  c->jit_n = 0;                                          // (nothing is native until the kernel runs)
  {
    std::lock_guard<SpinMutex> lk(c->prod_mu);
    __atomic_store_n(&c->bell->jit_gen, c->jit_gen, __ATOMIC_RELEASE);
    if (c->push) _mm_sfence();
  }
  if (live) {
    const int rc = jit_launch(c);
    if (rc != GPUOS_OK) {
      // should it start after all it must leave at once: ask for a generation it is not
      std::lock_guard<SpinMutex> lk(c->prod_mu);
      __atomic_store_n(&c->bell->jit_gen, c->jit_gen + 1, __ATOMIC_RELEASE);
      bump_epoch(c, 0xff, false);
      c->jit_failed = true;
      c->jit_error = std::string("the run-time worker kernel did not start: ") + gpuos_strerror(rc);
      return;
    }
    c->jit_n = n;
    jit_set_native(c, 1, true);
  } else {
    c->jit_n = n;                                        // gpuos_start_worker launches it and raises the flags
  }
}

}  // namespace

int gpuos_define_program(gpuos_ctx* c, const gpuos_instr* code, uint32_t n_instr, uint32_t n_inputs, uint32_t* out_impl_id) {
  if (!c || !code || !out_impl_id) return GPUOS_E_INVAL;
  if (n_instr < 1 || n_instr > GPUOS_PROGRAM_MAX_INSTR || n_inputs < 1 || n_inputs > GPUOS_MAX_INPUTS) return GPUOS_E_INVAL;
  ProgramImage img;
  std::memset(&img, 0, sizeof(img));
  for (uint32_t i = 0; i < n_instr; ++i) {
    const gpuos_instr& in = code[i];
    if (in.op >= GPUOS_PC_COUNT || in.dst >= GPUOS_PROGRAM_REGS || in.a >= GPUOS_PROGRAM_REGS || in.b >= GPUOS_PROGRAM_REGS)
      return GPUOS_E_INVAL;
    img.code[2 * i] = (uint32_t)in.op | ((uint32_t)in.dst << 8) | ((uint32_t)in.a << 16) | ((uint32_t)in.b << 24);
    std::memcpy(&img.code[2 * i + 1], &in.imm, 4);
  }
  img.n_instr = n_instr; img.n_inputs = n_inputs; img.ready = kProgramReady;
  {
    std::lock_guard<SpinMutex> lk(c->prod_mu);
    if (!c->worker_running && !c->worker_joined) return GPUOS_E_DEAD;
    if (c->n_progs >= GPUOS_MAX_PROGRAMS) return GPUOS_E_FULL;
    const uint32_t k = c->n_progs;
    // the code first, the header (with the ready word) after it: the device never runs half a program
    std::memcpy(c->progs[k].code, img.code, sizeof(img.code));
    if (c->push) _mm_sfence();
    std::atomic_thread_fence(std::memory_order_release);
    std::memcpy(&c->progs[k], &img, 16);
    if (c->push) _mm_sfence();
    std::atomic_thread_fence(std::memory_order_release);
    c->prog_img[k] = img;
    c->prog_arity[k] = (uint8_t)n_inputs;
    c->prog_len[k] = n_instr;
    uint64_t hsh = 0xcbf29ce484222325ull;                            // FNV-1a over the caller's instruction bytes
    for (size_t b = 0; b < (size_t)n_instr * sizeof(gpuos_instr); ++b)
      hsh = (hsh ^ reinterpret_cast<const unsigned char*>(code)[b]) * 0x100000001b3ull;
    c->prog_hash[k] = hsh;
    c->n_progs = k + 1;
    *out_impl_id = GPUOS_IMPL_PROGRAM_BASE + k;
    audit(c, GPUOS_AUDIT_DEFINE_PROGRAM, 0, GPUOS_IMPL_PROGRAM_BASE + k, 0);
  }
  // The program is usable (interpreted) from here.  Its native code is built when an operator is
  // first bound to it (gpuos_register_op / gpuos_swap_op), one kernel for all programs defined by
  // then; with cfg.jit_mode = 1, here.
  if (c->cfg.jit_mode == 1) jit_install(c);
  return GPUOS_OK;
}

namespace {
// Binding an operator to a program whose native code is not live yet: compile, in the calling thread
// and outside the producers' lock, a worker kernel for all programs defined so far, and bring it up
// (the program is interpreted until then, and for good if this fails).
void jit_before_bind(gpuos_ctx* c, uint32_t impl_id) {
  if (impl_id < GPUOS_IMPL_PROGRAM_BASE || !c->jit_enabled || c->jit_failed) return;
  bool need;
  {
    std::lock_guard<SpinMutex> lk(c->prod_mu);
    const uint32_t k = impl_id - GPUOS_IMPL_PROGRAM_BASE;
    need = k < c->n_progs && (k >= c->jit_n || !c->jit_mod);
  }
  if (need) jit_install(c);
}
}  // namespace

int gpuos_register_op(gpuos_ctx* c, uint32_t op_id, uint32_t impl_id, uint32_t* out_version) {
  if (!c || op_id >= GPUOS_MAX_OPS) return GPUOS_E_INVAL;
  if (impl_id == GPUOS_IMPL_NONE || (impl_id >= GPUOS_IMPL_COUNT && impl_id < GPUOS_IMPL_PROGRAM_BASE)) return GPUOS_E_BADOP;
  jit_before_bind(c, impl_id);
  std::lock_guard<SpinMutex> lk(c->prod_mu);
  if (!impl_known(c, impl_id)) return GPUOS_E_BADOP;
  if (c->ops[op_id].version != 0) return GPUOS_E_INVAL;            // already bound: use swap_op
  if (!c->worker_running && !c->worker_joined) return GPUOS_E_DEAD;   // a stopped worker reads the table when it is started again
  OpInfo& o = c->ops[op_id];
  __atomic_store_n(&o.impl, impl_id, __ATOMIC_RELAXED);
  __atomic_store_n(&o.version, 1u, __ATOMIC_RELEASE);
  o.prev_swap_head = 0;
  __atomic_store_n(&c->htable[op_id].slot[1], pack_entry(impl_id, 1), __ATOMIC_RELAXED);
  if (c->push) _mm_sfence();                 // write-combined stores: the slot before the version
  __atomic_store_n(&c->htable[op_id].version, 1u, __ATOMIC_RELEASE);
  bump_epoch(c, op_id, false);
  audit(c, GPUOS_AUDIT_REGISTER, op_id, impl_id, 1);
  if (out_version) *out_version = 1;
  return GPUOS_OK;
}

int gpuos_swap_op(gpuos_ctx* c, uint32_t op_id, uint32_t impl_id, uint32_t* out_version) {
  if (!c || op_id >= GPUOS_MAX_OPS) return GPUOS_E_INVAL;
  jit_before_bind(c, impl_id);
  std::lock_guard<SpinMutex> lk(c->prod_mu);
  if (!impl_known(c, impl_id)) return GPUOS_E_BADOP;
  OpInfo& o = c->ops[op_id];
  if (o.version == 0) return GPUOS_E_BADOP;
  if (!c->worker_running && !c->worker_joined) return GPUOS_E_DEAD;
  if (impl_id != GPUOS_IMPL_FAIL && o.impl != GPUOS_IMPL_FAIL &&
      (ctx_impl_arity(c, impl_id) != ctx_impl_arity(c, o.impl) || impl_kind(impl_id) != impl_kind(o.impl)))
    return GPUOS_E_INVAL;
  // The inactive slot still holds version-1's predecessor.  A task can only hold
  // that entry if it was submitted before the previous swap returned: wait for those.
  if (o.prev_swap_head > c->floor.load(std::memory_order_acquire)) {
    doorbell(c);
    const int rc = wait_floor(c, o.prev_swap_head, c->wait_ns);
    if (rc != GPUOS_OK) return rc;
  }
  const uint32_t v = o.version + 1;
  __atomic_store_n(&c->htable[op_id].slot[v & 1u], pack_entry(impl_id, v), __ATOMIC_RELAXED);  // inactive slot
  if (c->push) _mm_sfence();                 // write-combined stores: the slot before the version
  __atomic_store_n(&c->htable[op_id].version, v, __ATOMIC_RELEASE);                           // flip
  bump_epoch(c, op_id, false);
  __atomic_store_n(&o.impl, impl_id, __ATOMIC_RELAXED);
  __atomic_store_n(&o.version, v, __ATOMIC_RELEASE);
  o.prev_swap_head = c->head.load(std::memory_order_relaxed);
  audit(c, impl_id == GPUOS_IMPL_FAIL ? GPUOS_AUDIT_KILL : GPUOS_AUDIT_SWAP, op_id, impl_id, v);
  if (out_version) *out_version = v;
  return GPUOS_OK;
}

namespace {
int submit_impl(gpuos_ctx* c, const gpuos_task* tasks, uint32_t n, uint64_t* out_first_ticket, bool publish);
}
int gpuos_submit(gpuos_ctx* c, const gpuos_task* tasks, uint32_t n, uint64_t* out_first_ticket) {
  return submit_impl(c, tasks, n, out_first_ticket, false);
}
int gpuos_submit_flush(gpuos_ctx* c, const gpuos_task* tasks, uint32_t n, uint64_t* out_first_ticket) {
  return submit_impl(c, tasks, n, out_first_ticket, true);
}
namespace {
int submit_impl(gpuos_ctx* c, const gpuos_task* tasks, uint32_t n, uint64_t* out_first_ticket, bool publish) {
  if (!c || (!tasks && n)) return GPUOS_E_INVAL;
  if (!c->worker_running || worker_exited(c)) return GPUOS_E_DEAD;
  MarkerRange mr(c->cfg.markers != 0, "gpuos_submit %llu tasks", n);
  if (n == 0) {
    if (out_first_ticket) *out_first_ticket = c->head.load(std::memory_order_acquire);
    if (publish) doorbell_locked(c);
    return GPUOS_OK;
  }
  // pass 1 (no shared state: any number of host threads do this side by side): validate
  // everything and pack it; nothing is enqueued if one descriptor fails validation (a blocking
  // submit that runs out of time waiting for room keeps what it has enqueued: see the header)
  static thread_local std::vector<Record> staged;
  try {
    staged.resize(n);
  } catch (const std::bad_alloc&) {                             // no exception may cross the C boundary
    return GPUOS_E_NOMEM;
  }
  for (uint32_t i = 0; i < n; ++i) {
    const gpuos_task& t = tasks[i];
    uint32_t impl = GPUOS_IMPL_NONE;
    if (t.op_id < GPUOS_MAX_OPS && __atomic_load_n(&c->ops[t.op_id].version, __ATOMIC_ACQUIRE) != 0)
      impl = __atomic_load_n(&c->ops[t.op_id].impl, __ATOMIC_RELAXED);
    int rc;
    if (impl == GPUOS_IMPL_NONE) {
      if (!c->cfg.defer_op_check) return GPUOS_E_BADOP;
      rc = pack_task(t, GPUOS_IMPL_FAIL, &staged[i], c->cfg.chunk_elems);   // the device reports the bad op id
    } else {
      // a program's arity was stored before its id could be bound to any operator
      const int pa = impl >= GPUOS_IMPL_PROGRAM_BASE ? (int)c->prog_arity[(impl - GPUOS_IMPL_PROGRAM_BASE) % GPUOS_MAX_PROGRAMS] : 0;
      rc = pack_task(t, impl, &staged[i], c->cfg.chunk_elems, pa);
    }
    if (rc != GPUOS_OK) return rc;
    for (int k = 0; k < 3; ++k)
      if (t.dep[k] >= c->cap) return GPUOS_E_INVAL;
    // The part of the check word that does not depend on the ticket: the weighted sum of the
    // other 63 words, with the record's ticket field zero (the ticket enters through the seed only).
    staged[i].ticket = 0;
    staged[i].check = record_check_sum(reinterpret_cast<const uint32_t*>(&staged[i]), 63);
  }
  // pass 2 (one producer at a time): reserve n consecutive tickets and write the records
  std::lock_guard<SpinMutex> lk(c->prod_mu);
  uint64_t head = c->head.load(std::memory_order_relaxed);
  for (uint32_t i = 0; i < n; ++i)
    for (int k = 0; k < 3; ++k)
      if (tasks[i].dep[k] > head + i) return GPUOS_E_INVAL;       // names a ticket before the first one
  if (out_first_ticket) *out_first_ticket = head;
  const bool direct = publish && n == 1 && c->direct_store;
  if (c->cfg.nonblocking_submit) {
    if (!c->harvester_run.load(std::memory_order_relaxed)) harvest(c);
    if ((uint64_t)n > c->cap - (head - c->floor.load(std::memory_order_acquire))) return GPUOS_E_FULL;
  }
  for (uint32_t i = 0; i < n; ++i) {
    if (head - c->floor.load(std::memory_order_acquire) >= c->cap) {
      c->head.store(head, std::memory_order_release);
      doorbell(c);                                                // publish so that the device can make room
      const int rc = wait_floor(c, head - c->cap + 1, c->wait_ns);
      if (rc != GPUOS_OK) return rc;
    }
    Record& rec = staged[i];
    rec.check = record_check_seed(head) - rec.check;              // pass 1 left the sum of the other 63 words here
    if (direct) direct_store_record(&c->hring[head & c->mask], &rec);
    else std::memcpy(&c->hring[head & c->mask], &rec, sizeof(Record));
    ++head;
  }
  if (publish) {
    // a lone record and the doorbell leave this core with one flush of its write-combining buffers,
    // or, as direct stores, with none
    c->head.store(head, std::memory_order_release);
    doorbell(c, n > 1, direct);
    return GPUOS_OK;
  }
  // Device-memory ring: the records sit in THIS core's write-combining buffers; push them out
  // before another producer thread can ring the doorbell over them.
  if (c->push) _mm_sfence();
  c->head.store(head, std::memory_order_release);
  return GPUOS_OK;
}
}  // namespace

int gpuos_flush(gpuos_ctx* c) {
  if (!c) return GPUOS_E_INVAL;
  if (!c->worker_running) return GPUOS_E_DEAD;
  doorbell_locked(c);
  return GPUOS_OK;
}

int gpuos_wait(gpuos_ctx* c, uint64_t ticket, uint64_t timeout_ns) {
  if (!c) return GPUOS_E_INVAL;
  MarkerRange mr(c->cfg.markers != 0, ticket == GPUOS_ALL ? "gpuos_wait all" : "gpuos_wait ticket %llu", ticket);
  if (c->worker_running) doorbell_locked(c);
  const bool all = ticket == GPUOS_ALL;
  const uint64_t head = c->head.load(std::memory_order_acquire);
  if (!all && ticket >= head) return GPUOS_E_INVAL;
  const uint64_t target = all ? head : ticket + 1;
  if (c->floor.load(std::memory_order_acquire) < target) {
    if (!c->worker_running) return GPUOS_E_DEAD;
    const int rc = wait_floor(c, target, timeout_ns ? timeout_ns : c->wait_ns);
    if (rc != GPUOS_OK) return rc;
  }
  if (all) return c->first_error.exchange(0);
  if (head - ticket > c->log_mask + 1) return GPUOS_OK;           // fell out of the log
  return c->log[ticket & c->log_mask].status;
}

int gpuos_get_completions(gpuos_ctx* c, uint64_t first, uint32_t n, gpuos_completion* out) {
  if (!c || (!out && n)) return GPUOS_E_INVAL;
  const uint64_t fl = c->floor.load(std::memory_order_acquire);
  if (first + n > fl) return GPUOS_E_INVAL;
  if (fl - first > c->log_mask + 1) return GPUOS_E_INVAL;
  for (uint32_t i = 0; i < n; ++i) out[i] = c->log[(first + i) & c->log_mask];
  return GPUOS_OK;
}

int gpuos_peek_queue(gpuos_ctx* c, gpuos_queue_state* out) {
  if (!c || !out) return GPUOS_E_INVAL;
  if (c->worker_running && !c->harvester_run.load(std::memory_order_relaxed)) harvest(c);
  out->head_submitted = c->head.load(std::memory_order_acquire);
  out->tail_published = c->published.load(std::memory_order_acquire);
  out->claimed = c->h ? __atomic_load_n(&c->h->dispatched, __ATOMIC_ACQUIRE) : 0;
  out->completed = c->floor.load(std::memory_order_acquire);
  out->heartbeat = c->h ? __atomic_load_n(&c->h->heartbeat, __ATOMIC_ACQUIRE) : 0;
  out->capacity = c->cap;
  out->workgroups = c->workgroups;
  out->push_ring = c->push ? 1u : 0u;
  out->reserved = 0;
  return GPUOS_OK;
}

int gpuos_worker_alive(gpuos_ctx* c) {
  if (!c || !c->worker_running || !c->h) return 0;
  if (worker_exited(c)) return 0;
  // the dispatcher bumps the heartbeat every 64 polls (a few hundred microseconds at most)
  const uint64_t hb0 = __atomic_load_n(&c->h->heartbeat, __ATOMIC_ACQUIRE);
  const uint64_t t0 = now_ns();
  while (now_ns() - t0 < 50000000ull) {
    if (__atomic_load_n(&c->h->heartbeat, __ATOMIC_ACQUIRE) != hb0) return 1;
    if (hipStreamQuery(c->stream) != hipErrorNotReady) return 0;
  }
  // no poll for 50 ms: the dispatcher may be busy mirroring; the kernel is still resident
  return hipStreamQuery(c->stream) == hipErrorNotReady ? 1 : 0;
}

int gpuos_set_yield_every(gpuos_ctx* c, uint32_t every) {
  if (!c) return GPUOS_E_INVAL;
  if (!c->worker_running) return GPUOS_E_DEAD;
  std::lock_guard<SpinMutex> lk(c->prod_mu);                      // the epoch is the producers' (a swap may be running)
  __atomic_store_n(&c->bell->yield_every, every, __ATOMIC_RELEASE);
  bump_epoch(c, 0xff, false);
  return GPUOS_OK;
}

int gpuos_stop_worker(gpuos_ctx* c) {
  if (!c) return GPUOS_E_INVAL;
  MarkerRange mr(c->cfg.markers != 0, "gpuos_stop_worker");
  return stop_worker(c);
}

int gpuos_start_worker(gpuos_ctx* c) {
  if (!c || !c->h) return GPUOS_E_INVAL;
  if (c->worker_running && !worker_exited(c)) return GPUOS_OK;          // it is running
  if (c->worker_running) {                                              // it left by itself (idle exit): join it
    const int rc = stop_worker(c);
    if (rc != GPUOS_OK) return rc;
  }
  if (!c->worker_joined) return GPUOS_E_DEAD;                           // an earlier stop timed out: the kernel may still be there
  // A worker that leaves drains what it has dequeued.  Records published after its last look at the
  // doorbell (an idle exit can race with a submit) are still in the ring: the new worker takes them.
  const uint64_t head = __atomic_load_n(&c->h->dispatched, __ATOMIC_ACQUIRE);
  if (c->floor.load(std::memory_order_acquire) != head) return GPUOS_E_DEAD;   // dequeued work was lost: not a state to continue from
  HIP_TRY(hipSetDevice(c->device));
  __atomic_store_n(&c->h->exit_code, 0u, __ATOMIC_RELEASE);
  __atomic_store_n(&c->h->heartbeat, (uint64_t)0, __ATOMIC_RELEASE);
  {
    std::lock_guard<SpinMutex> lk(c->prod_mu);
    bump_epoch(c, 0xff, false);                                         // lowers the stop bit; the new worker reads the whole table
  }
  WorkerArgs a = c->wargs;
  a.resume = 1;
  a.resume_tickets = head;
  HIP_TRY((hipError_t)launch_resume_fixup(c->d, c->stream));
  if (c->ev_start) HIP_TRY(hipEventRecord(c->ev_start, c->stream));
  HIP_TRY((hipError_t)launch_worker(a, c->workgroups, c->stream));
  if (c->ev_stop) HIP_TRY(hipEventRecord(c->ev_stop, c->stream));
  c->worker_running = true;
  c->worker_joined = false;
  const uint64_t t0 = now_ns();
  uint32_t spins = 0;
  while (__atomic_load_n(&c->h->heartbeat, __ATOMIC_ACQUIRE) == 0) {
    if ((spins & 255u) == 0 && now_ns() - t0 > c->wait_ns) {
      (void)stop_worker(c);                                             // leaves as soon as it starts
      return GPUOS_E_TIMEOUT;
    }
    if ((++spins & 4095u) == 0 && hipStreamQuery(c->stream) != hipErrorNotReady) {
      c->worker_running = false; c->worker_joined = true;
      return GPUOS_E_DEAD;
    }
    __builtin_ia32_pause();
  }
  if (c->cfg.harvester_thread) {
    c->harvester_run.store(true);
    c->harvester = std::thread(harvester_main, c, sched_getcpu());
  }
  if (c->jit_enabled && !c->jit_failed && c->jit_mod && c->jit_n) {   // the native code of the programs comes back too
    std::lock_guard<std::mutex> jl(c->jit_mu);
    const int rc = jit_launch(c);
    if (rc == GPUOS_OK) jit_set_native(c, 1, true);
    else {
      std::lock_guard<SpinMutex> lk(c->prod_mu);
      __atomic_store_n(&c->bell->jit_gen, c->jit_gen + 1, __ATOMIC_RELEASE);     // should it start after all, it leaves at once
      bump_epoch(c, 0xff, false);
      c->jit_failed = true;
      c->jit_error = std::string("the run-time worker kernel did not start again: ") + gpuos_strerror(rc);
    }
  }
  marker(c->cfg.markers != 0, "gpuos: worker launched again at ticket %llu", head);
  return GPUOS_OK;
}

int gpuos_worker_elapsed_ms(gpuos_ctx* c, float* out_ms) {
  if (!c || !out_ms) return GPUOS_E_INVAL;
  if (!c->worker_joined || !c->ev_start) return GPUOS_E_INVAL;   // (a static context has no events)
  HIP_TRY(hipEventElapsedTime(out_ms, c->ev_start, c->ev_stop));
  return GPUOS_OK;
}

int gpuos_worker_stats(gpuos_ctx* c, uint64_t out[16]) {
  if (!c || !out) return GPUOS_E_INVAL;
  if (!c->worker_joined) return GPUOS_E_INVAL;
  HIP_TRY(hipSetDevice(c->device));
  HIP_TRY(hipMemcpy(out, c->d->stat, sizeof(uint64_t) * 16, hipMemcpyDeviceToHost));
  return GPUOS_OK;
}

int gpuos_native_info(gpuos_ctx* c, uint64_t out[8], char* why, uint32_t why_len) {
  if (!c || !out) return GPUOS_E_INVAL;
  std::lock_guard<std::mutex> jl(c->jit_mu);
  out[0] = (c->jit_enabled && !c->jit_failed && c->jit_running) ? 1u : 0u;
  out[1] = c->jit_gen;
  out[2] = out[0] ? c->jit_n : 0u;
  out[3] = c->jit_builds;
  out[4] = c->jit_cache_hits;
  out[5] = 0;
  out[6] = (uint64_t)(c->jit_last_ms * 1000.0);
  out[7] = c->jit_grid;
  if (c->worker_joined && c->d && !c->static_mode) {                    // device counters are read once the kernels have left
    HIP_TRY(hipSetDevice(c->device));
    HIP_TRY(hipMemcpy(&out[5], &c->d->jit_units, sizeof(uint64_t), hipMemcpyDeviceToHost));
    out[0] = (c->jit_enabled && !c->jit_failed && c->jit_mod) ? 1u : 0u;
    out[2] = out[0] ? c->jit_n : 0u;
  }
  if (why && why_len) {
    std::strncpy(why, c->jit_error.c_str(), why_len - 1);
    why[why_len - 1] = 0;
  }
  return GPUOS_OK;
}

int gpuos_shutdown(gpuos_ctx* c) {
  if (!c) return GPUOS_OK;
  const int rc = stop_worker(c);
  {
    std::lock_guard<std::mutex> lk(g_live_mu);
    for (size_t i = 0; i < g_live.size(); ++i)
      if (g_live[i] == c) { g_live.erase(g_live.begin() + (long)i); break; }
  }
  if (!c->worker_joined) return rc;         // the kernel may still be running: leak rather than free under it
  (void)hipSetDevice(c->device);
  if (c->static_mode) {                     // the caller's block and stream; the device array goes back to the pool of one
    const int dev = c->device;
    c->~gpuos_ctx();
    g_static_owner[dev].store(nullptr);
    return rc;
  }
  free_all(c);
  delete c;
  return rc;
}

int gpuos_run_serial(gpuos_ctx* c, const gpuos_task* tasks, uint32_t n, uint64_t* lat_ns) {
  if (!c || (!tasks && n)) return GPUOS_E_INVAL;
  for (uint32_t i = 0; i < n; ++i) {
    const uint64_t t0 = now_ns();
    uint64_t ticket = 0;
    int rc = gpuos_submit_flush(c, &tasks[i], 1, &ticket);
    if (rc == GPUOS_OK) rc = gpuos_wait(c, ticket, 0);
    if (rc != GPUOS_OK) return rc;
    if (lat_ns) lat_ns[i] = now_ns() - t0;
  }
  return GPUOS_OK;
}

int gpuos_launch_per_op(int32_t device, const gpuos_task* tasks, uint32_t n, const uint32_t* impl_of_op,
                        int32_t sync_each, uint64_t* lat_ns, double* out_seconds) {
  if ((!tasks && n) || !impl_of_op) return GPUOS_E_INVAL;
  HIP_TRY(hipSetDevice(device));
  hipStream_t s;
  HIP_TRY(hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
  int rc = GPUOS_OK;
  const uint64_t t0 = now_ns();
  for (uint32_t i = 0; i < n && rc == GPUOS_OK; ++i) {
    const uint64_t ta = sync_each ? now_ns() : 0;
    Record r;
    const uint32_t impl = tasks[i].op_id < GPUOS_MAX_OPS ? impl_of_op[tasks[i].op_id] : 0u;
    if (impl == GPUOS_IMPL_NONE) { rc = GPUOS_E_BADOP; break; }
    rc = pack_task(tasks[i], impl, &r);
    if (rc != GPUOS_OK) break;
    if (r.path != PATH_NOP && !hip_ok((hipError_t)launch_single(r, s), "launch per op")) { rc = GPUOS_E_HIP; break; }
    if (sync_each) {
      if (!hip_ok(hipStreamSynchronize(s), "hipStreamSynchronize")) { rc = GPUOS_E_HIP; break; }
      if (lat_ns) lat_ns[i] = now_ns() - ta;
    }
  }
  if (!hip_ok(hipStreamSynchronize(s), "hipStreamSynchronize") && rc == GPUOS_OK) rc = GPUOS_E_HIP;
  if (out_seconds) *out_seconds = (double)(now_ns() - t0) * 1e-9;
  (void)hipStreamDestroy(s);
  return rc;
}

int gpuos_submit_from_threads(gpuos_ctx* c, const gpuos_task* tasks, uint32_t n, uint32_t n_threads,
                              uint32_t batch, uint32_t passes, double* out_seconds) {
  if (!c || (!tasks && n) || n_threads == 0 || n_threads > 256 || batch == 0) return GPUOS_E_INVAL;
  if (n_threads == 1) {
    const uint64_t t0 = now_ns();
    int rc = GPUOS_OK;
    for (uint32_t p = 0; p < passes && rc == GPUOS_OK; ++p)
      for (uint32_t i = 0; i < n && rc == GPUOS_OK; i += batch) {
        rc = gpuos_submit_flush(c, tasks + i, n - i < batch ? n - i : batch, nullptr);
      }
    if (out_seconds) *out_seconds = (double)(now_ns() - t0) * 1e-9;
    return rc;
  }
  std::vector<std::thread> threads;
  std::vector<int> rcs(n_threads, GPUOS_OK);
  std::atomic<uint32_t> ready{0};
  std::atomic<bool> go{false};
  for (uint32_t k = 0; k < n_threads; ++k) {
    threads.emplace_back([&, k] {
      const uint32_t lo = (uint32_t)((uint64_t)k * n / n_threads), hi = (uint32_t)((uint64_t)(k + 1) * n / n_threads);
      ready.fetch_add(1);
      while (!go.load(std::memory_order_acquire)) __builtin_ia32_pause();
      for (uint32_t p = 0; p < passes && rcs[k] == GPUOS_OK; ++p)
        for (uint32_t i = lo; i < hi && rcs[k] == GPUOS_OK; i += batch) {
          rcs[k] = gpuos_submit_flush(c, tasks + i, hi - i < batch ? hi - i : batch, nullptr);
        }
    });
  }
  while (ready.load() < n_threads) __builtin_ia32_pause();
  const uint64_t t0 = now_ns();
  go.store(true, std::memory_order_release);
  for (auto& t : threads) t.join();
  if (out_seconds) *out_seconds = (double)(now_ns() - t0) * 1e-9;
  for (int rc : rcs) if (rc != GPUOS_OK) return rc;
  return GPUOS_OK;
}

int gpuos_get_trace(gpuos_ctx* c, uint64_t first, uint32_t n, gpuos_trace_record* out) {
  if (!c || !out || !c->trace) return GPUOS_E_INVAL;
  static_assert(sizeof(gpuos_trace_record) == sizeof(TraceRec), "trace record layout");
  if (first + n > c->floor.load(std::memory_order_acquire)) {
    if (c->worker_running && !c->harvester_run.load(std::memory_order_relaxed)) harvest(c);
    if (first + n > c->floor.load(std::memory_order_acquire)) return GPUOS_E_INVAL;   // not complete yet
  }
  for (uint32_t i = 0; i < n; ++i) {
    const TraceRec* tr = &c->trace[(first + i) & c->trace_mask];
    std::memcpy(&out[i], tr, sizeof(TraceRec));
    if (out[i].ticket != first + i) return GPUOS_E_INVAL;      // overwritten by a later ticket
  }
  return GPUOS_OK;
}

int gpuos_op_counts(gpuos_ctx* c, uint64_t* out) {
  if (!c || !out || !c->opcount) return GPUOS_E_INVAL;
  for (uint32_t op = 0; op < GPUOS_MAX_OPS; ++op) out[op] = __atomic_load_n(&c->opcount[op], __ATOMIC_ACQUIRE);
  return GPUOS_OK;
}

int gpuos_trace_origin(gpuos_ctx* c, uint64_t* host_ns) {
  if (!c || !host_ns || !c->trace) return GPUOS_E_INVAL;
  *host_ns = c->origin_host_ns;
  return GPUOS_OK;
}

int gpuos_kill_op(gpuos_ctx* c, uint32_t op_id, uint32_t* out_version) {
  return gpuos_swap_op(c, op_id, GPUOS_IMPL_FAIL, out_version);
}

int gpuos_audit_log(gpuos_ctx* c, uint64_t first, uint32_t n, gpuos_audit_record* out, uint64_t* out_total) {
  if (!c || (!out && n)) return GPUOS_E_INVAL;
  std::lock_guard<SpinMutex> lk(c->prod_mu);
  if (out_total) *out_total = c->audit_total;
  const uint64_t oldest = c->audit_total - c->audit.size();
  if (first < oldest || first + n > c->audit_total) return GPUOS_E_INVAL;
  for (uint32_t i = 0; i < n; ++i) out[i] = c->audit[(size_t)((first + i) % kAuditKeep)];   // record k lives at k mod kAuditKeep
  return GPUOS_OK;
}

int gpuos_task_plan(const gpuos_task* t, uint32_t impl, uint32_t out[4]) {
  if (!t || !out) return GPUOS_E_INVAL;
  Record r;
  const int rc = pack_task(*t, impl, &r);
  if (rc != GPUOS_OK) return rc;
  out[0] = r.path; out[1] = r.nchunks; out[2] = r.chunk; out[3] = r.ndim;
  return GPUOS_OK;
}

int gpuos_task_bytes(const gpuos_task* t, uint32_t impl, uint64_t* out_bytes) {
  if (!t || !out_bytes) return GPUOS_E_INVAL;
  Record r;
  const int rc = pack_task(*t, impl, &r);
  if (rc != GPUOS_OK) return rc;
  *out_bytes = 0;
  if (impl == GPUOS_IMPL_FAIL) return GPUOS_OK;
  const int ar = impl_arity(impl);
  const bool red = impl_is_reduction(impl);
  uint64_t out_elems = 1;
  for (int d = 0; d < (red ? t->ndim - 1 : t->ndim); ++d) out_elems *= (uint64_t)t->size[d];
  uint64_t total = out_elems * dtype_size(t->out.dtype);
  for (int k = 0; k < ar; ++k) {
    uint64_t distinct = 1;
    for (int d = 0; d < t->ndim; ++d) {
      const bool bc = ((t->in[k].bcast_mask >> d) & 1) || t->in[k].stride[d] == 0;
      if (!bc) distinct *= (uint64_t)t->size[d];
      else if (t->size[d] == 0) distinct = 0;
    }
    total += distinct * dtype_size(t->in[k].dtype);
  }
  *out_bytes = total;
  return GPUOS_OK;
}

const char* gpuos_strerror(int status) {
  switch (status) {
    case GPUOS_OK: return "ok";
    case GPUOS_E_INVAL: return "invalid argument or descriptor";
    case GPUOS_E_FULL: return "ring full";
    case GPUOS_E_BADOP: return "unknown, unregistered or failed operator";
    case GPUOS_E_TIMEOUT: return "timed out";
    case GPUOS_E_DEAD: return "worker kernel is not running";
    case GPUOS_E_HIP: return "HIP runtime error";
    case GPUOS_E_NOMEM: return "out of memory";
    case GPUOS_E_VERSION: return "operator-table version mismatch";
    default: return "unknown status";
  }
}

int gpuos_device_info(int32_t device, uint64_t out[8], char* name, uint32_t name_len) {
  if (!out) return GPUOS_E_INVAL;
  hipDeviceProp_t p;
  HIP_TRY(hipGetDeviceProperties(&p, device));
  out[0] = (uint64_t)p.multiProcessorCount;
  out[1] = (uint64_t)p.clockRate;
  out[2] = (uint64_t)p.memoryClockRate;
  out[3] = (uint64_t)p.memoryBusWidth;
  out[4] = (uint64_t)p.totalGlobalMem;
  out[5] = (uint64_t)p.l2CacheSize;
  out[6] = (uint64_t)p.sharedMemPerBlock;
  out[7] = (uint64_t)p.warpSize;
  if (name && name_len) {
    std::strncpy(name, p.name, name_len - 1);
    name[name_len - 1] = 0;
  }
  return GPUOS_OK;
}

const char* gpuos_last_hip_error(void) { return g_hip_error.c_str(); }

void gpuos_abi_layout(uint32_t out[8]) {
  out[0] = (uint32_t)sizeof(gpuos_task);
  out[1] = (uint32_t)sizeof(gpuos_tensor);
  out[2] = (uint32_t)offsetof(gpuos_task, size);
  out[3] = (uint32_t)offsetof(gpuos_task, in);
  out[4] = (uint32_t)offsetof(gpuos_task, out);
  out[5] = (uint32_t)offsetof(gpuos_task, alpha);
  out[6] = (uint32_t)offsetof(gpuos_task, dep);
  out[7] = (uint32_t)sizeof(gpuos_completion);
}

}  // extern "C"
