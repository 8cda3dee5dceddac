// Future/dispatch runtime and the C boundary (include/pw.h).
//
// Mapping of the paper's dispatch design onto one GPU:
//   compiled function (Section 3, App. B)  -> FnRec: kind + static signature + params, checked at compile time
//   buffer future (Section 4.4)            -> FutureRec: device buffer + HIP event + poison words + refcount
//   FIFO executor (Section 4.4)            -> one HIP stream; enqueue order is execution order
//   parallel asynchronous dispatch (4.5)   -> pw_chain validates and enqueues every function of the chain
//                                             before any input exists; output buffers come from a pool, so no
//                                             allocation or synchronisation sits between launches
//   one message per subgraph (4.5)         -> PW_GRAPH: the chain's launches replayed as one HIP graph
//   sequential dispatch baseline (5.1)     -> PW_SEQUENTIAL
//   nodes on different executors (4.5, Fig. 4; measured in 5.1, Fig. 7) -> pw_pipeline: one HIP stream and one
//                                             host thread per executor, dependencies carried by HIP events,
//                                             a copy into the consumer's pre-allocated buffer as the transfer
//   device object store (4.6)              -> handle tables + size-class buffer pool + refcounts
// An input that "is not ready" is made real by a gate kernel on a second stream that spins (bounded) on a
// word in pinned host memory; consumers wait on the event recorded behind it.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <deque>
#include <map>
#include <mutex>
#include <thread>
#include <memory>
#include <string>
#include <unordered_map>
#include <vector>

#include "../../include/pw.h"
#include "kernels.hpp"
#include "encdec.hpp"
#include "lm.hpp"

using namespace pw;

namespace {

size_t dtype_size(int dt) { return dt == PW_BF16 ? 2 : 4; }

bool spec_ok(const pw_tensor_spec& s) {
  if (s.dtype < PW_F32 || s.dtype > PW_I32 || s.rank < 0 || s.rank > 4) return false;
  for (int i = 0; i < s.rank; ++i)
    if (s.dims[i] < 0 || s.dims[i] > (1LL << 40)) return false;
  return true;
}
int64_t spec_numel(const pw_tensor_spec& s) {
  int64_t n = 1;
  for (int i = 0; i < s.rank; ++i) n *= s.dims[i];
  return n;
}
size_t spec_bytes(const pw_tensor_spec& s) { return (size_t)spec_numel(s) * dtype_size(s.dtype); }
// 0 same, PW_ERR_DTYPE or PW_ERR_SHAPE otherwise
pw_status spec_match(const pw_tensor_spec& a, const pw_tensor_spec& b) {
  if (a.dtype != b.dtype) return PW_ERR_DTYPE;
  if (a.rank != b.rank) return PW_ERR_SHAPE;
  for (int i = 0; i < a.rank; ++i)
    if (a.dims[i] != b.dims[i]) return PW_ERR_SHAPE;
  return PW_OK;
}

// A pair of words in pinned host memory: [0] the gate flag the host sets, [1] the poison mark.
struct GateWords {
  uint32_t* words;   // host-visible, device-visible
};

struct FutureRec {
  bool live = false;
  uint32_t gen = 0;
  void* buf = nullptr;
  size_t bytes = 0, pool_bytes = 0;
  pw_tensor_spec spec{};
  bool owns = false;             // buffer goes back to the pool on release
  bool on_gate_stream = false;   // produced by the gate stream: consumers must wait on `event`
  bool pending = false;          // created by pw_future_pending and not resolved yet
  hipEvent_t event = nullptr;    // null: ready w.r.t. the executor stream's order
  int refcount = 0;
  uint64_t owner = 0;            // ownership label (Section 4.6): who this object dies with
  bool host_poison = false;
  std::vector<std::shared_ptr<GateWords>> poison;   // gates this future depends on
  std::shared_ptr<GateWords> gate;                  // own gate (pending futures)
  void* staging = nullptr;                          // pinned host staging (pending futures)
};

struct FnRec {
  bool live = false;
  uint32_t gen = 0;
  pw_fn_desc desc{};
  float cst = 0.f, busy_us = 0.f;
  int reps = 1;
  Model* model = nullptr;
  EncDec* encdec = nullptr;
  int microbatch = 0;
};

struct GraphEntry {
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
};

// One node of a pipeline as handed to an executor's host thread.  Everything the thread needs is in here (the
// controller planned every buffer beforehand: shapes are static), so the thread touches no context tables.
struct NodeMsg {
  int kind = 0;
  float cst = 0.f, busy_us = 0.f;
  int reps = 1;
  int64_t numel = 0;
  const float* in = nullptr;
  float* out = nullptr;
  void* xfer_dst = nullptr;          // consumer-side buffer on another executor (null: consumer shares this stream)
  size_t xfer_bytes = 0;
  hipEvent_t wait_event = nullptr;   // producer's event on another stream (null: none, or same stream)
  std::atomic<int>* wait_flag = nullptr;   // set by the producer's thread once wait_event has been recorded (1) or it failed (2)
  hipEvent_t done_event = nullptr;   // recorded behind this node (and its transfer)
  std::atomic<int>* done_flag = nullptr;
  std::atomic<int>* ack = nullptr;   // 1: enqueued, 2: failed
  int prep_us = 0;                   // emulated host-side preparation (see pw_ctx_set_executor_prep_us)
};

struct Executor {
  hipStream_t stream = nullptr;
  bool own_stream = false;
  std::thread thread;
  std::mutex mu;
  std::condition_variable cv;
  std::deque<NodeMsg> queue;
  bool stop = false;
};

}  // namespace

struct pw_sched;

struct pw_ctx {
  int device = 0;
  hipStream_t exec = nullptr;      // executor stream
  bool own_exec = false;
  hipStream_t gate = nullptr;      // gate kernels and their copies
  hipStream_t io = nullptr;        // device-to-host copies of pw_await
  std::string error;
  int gate_timeout_ms = 20000;

  std::vector<FutureRec> futures;
  std::vector<uint32_t> free_futures;
  std::vector<FnRec> fns;
  std::vector<Model*> models;
  std::vector<EncDec*> encdecs;
  int64_t live_futures = 0;
  uint64_t current_owner = 0;    // label given to futures created from now on
  int64_t memory_limit = 0;      // bytes the pool may have handed out at once; 0: no limit

  // buffer pool: power-of-two size classes
  std::map<size_t, std::vector<void*>> pool;
  int64_t pool_in_use = 0;
  std::vector<hipEvent_t> event_pool;

  // pinned host words for gates
  std::vector<uint32_t*> word_slabs;
  std::vector<uint32_t*> free_words;
  std::map<size_t, std::vector<void*>> staging_pool;

  std::unordered_map<std::string, GraphEntry> graphs;

  std::vector<std::unique_ptr<Executor>> executors;   // pw_ctx_set_executors; [0] wraps the executor stream
  int executor_prep_us = 0;

  // Serialises the dispatch calls (functions, futures, chains, pipelines, await) so that client threads and the
  // scheduler thread of pw_sched may share a context.  Recursive: some calls are built from others.
  std::recursive_mutex api_mu;
  std::vector<pw_sched*> scheds;
  std::vector<pw_program*> programs;
};

#define PW_API_LOCK(c)                                  \
  std::unique_lock<std::recursive_mutex> api_lk_;       \
  if (c) api_lk_ = std::unique_lock<std::recursive_mutex>((c)->api_mu)

struct pw_model {
  pw_ctx* ctx;
  Model* impl;
};
struct pw_encdec {
  pw_ctx* ctx;
  EncDec* impl;
};

// ---- traced dataflow programs (Section 3) ---------------------------------------------------------------
namespace {
struct ProgNode {
  FnRec fn;            // snapshot: the handle may be released after tracing
  pw_fn handle = 0;    // only part of the graph-cache key
  int n_in = 0, in[8] = {0};
  int first_out = 0;
};
}  // namespace
struct pw_program {
  pw_ctx* ctx = nullptr;
  int n_inputs = 0;
  std::vector<pw_tensor_spec> specs;   // per value
  std::vector<ProgNode> nodes;
  std::vector<int> outputs;
  std::vector<int> last_use;           // per value: last node that reads it; n_nodes if it is a program output; -1 if unused
  std::unordered_map<std::string, GraphEntry> graphs;
};

// ---- multi-tenant scheduler (Section 4.4 "centralized scheduler", Section 5.2) -----------------------------
// Clients (any threads) put programs - chains of compiled functions - into per-client queues; ONE scheduler
// thread decides the order in which programs reach the executor stream, so that order is consistent whatever
// the clients do.  FIFO takes programs in arrival order; proportional share takes, among the clients that have
// work queued, the one whose weighted device time consumed so far (estimated at enqueue) is smallest (stride
// scheduling).  Only a bounded number of programs is kept in flight on the device, so a client that arrives
// late is not stuck behind an arbitrarily long backlog of others.
namespace {
struct SchedProgram {
  std::vector<pw_fn> fns;
  pw_future in = 0;
  uint64_t ticket = 0, arrival = 0;
  double est_us = 0;
  int n_computations = 0;
};
struct SchedClient {
  double weight = 1, vtime = 0;
  uint64_t owner = 0;
  bool failed = false;
  std::deque<SchedProgram> queue;
  int64_t programs = 0, computations = 0;
  double device_ms = 0;
};
struct SchedResult {
  pw_status status = PW_OK;
  pw_future out = 0;
};
struct SchedInFlight {
  int client = 0;
  int n_computations = 0;
  hipEvent_t start = nullptr, stop = nullptr;
};
}  // namespace

struct pw_sched {
  pw_ctx* ctx = nullptr;
  int policy = PW_SCHED_FIFO;
  int window = 4;                       // programs in flight on the device at most
  std::mutex mu;
  std::condition_variable cv_work, cv_done;
  std::vector<SchedClient> clients;
  std::unordered_map<uint64_t, SchedResult> results;
  std::unordered_map<uint64_t, bool> outstanding;   // tickets handed out and not yet collected (value: someone is waiting)
  uint64_t next_ticket = 1, next_arrival = 1;
  int64_t queued = 0;
  std::deque<SchedInFlight> inflight;   // scheduler thread only
  std::vector<hipEvent_t> timing_events;
  hipEvent_t epoch = nullptr;           // recorded at creation: slices are reported relative to it
  std::vector<pw_sched_slice> trace;
  int collecting = 0;                   // results taken by pw_sched_wait whose futures are not released yet
  int64_t stalls = 0;                   // programs that had to wait for memory
  double stalled_ms = 0;
  uint64_t id = 0;
  bool stop = false, idle = true;
  std::thread thread;
};

namespace {

pw_status fail(pw_ctx* c, pw_status st, const char* fmt, ...) {
  if (c) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    c->error = buf;
  }
  return st;
}
#define PW_HIP(c, expr)                                                                          \
  do {                                                                                           \
    hipError_t e_ = (expr);                                                                      \
    if (e_ != hipSuccess) return fail(c, e_ == hipErrorOutOfMemory ? PW_ERR_OOM : PW_ERR_DEVICE, \
                                      "%s: %s", #expr, hipGetErrorString(e_));                   \
  } while (0)

size_t size_class(size_t bytes) {
  size_t c = 256;
  while (c < bytes) c <<= 1;
  return c;
}

pw_status pool_alloc(pw_ctx* c, size_t bytes, void** out, size_t* cls_out) {
  const size_t cls = size_class(bytes ? bytes : 1);
  if (c->memory_limit > 0 && c->pool_in_use + (int64_t)cls > c->memory_limit)
    return fail(c, PW_ERR_OOM, "memory budget: %lld bytes in use, %zu more asked for, limit %lld", (long long)c->pool_in_use, cls,
                (long long)c->memory_limit);
  auto& fl = c->pool[cls];
  if (!fl.empty()) {
    *out = fl.back();
    fl.pop_back();
  } else {
    hipError_t e = hipMalloc(out, cls);
    if (e != hipSuccess) return fail(c, PW_ERR_OOM, "hipMalloc(%zu): %s", cls, hipGetErrorString(e));
  }
  *cls_out = cls;
  c->pool_in_use += (int64_t)cls;
  return PW_OK;
}
void pool_free(pw_ctx* c, void* p, size_t cls) {
  c->pool[cls].push_back(p);
  c->pool_in_use -= (int64_t)cls;
}

pw_status event_get(pw_ctx* c, hipEvent_t* ev) {
  if (!c->event_pool.empty()) {
    *ev = c->event_pool.back();
    c->event_pool.pop_back();
    return PW_OK;
  }
  PW_HIP(c, hipEventCreateWithFlags(ev, hipEventDisableTiming));
  return PW_OK;
}

std::shared_ptr<GateWords> words_get(pw_ctx* c) {
  if (c->free_words.empty()) {
    uint32_t* slab = nullptr;
    if (hipHostMalloc((void**)&slab, 4096, hipHostMallocDefault) != hipSuccess) return nullptr;
    c->word_slabs.push_back(slab);
    for (int i = 0; i < 4096 / 64; ++i) c->free_words.push_back(slab + i * 16);   // one 64-byte line per gate
  }
  uint32_t* w = c->free_words.back();
  c->free_words.pop_back();
  w[0] = 0;
  w[1] = 0;
  pw_ctx* ctx = c;
  return std::shared_ptr<GateWords>(new GateWords{w}, [ctx](GateWords* g) {
    ctx->free_words.push_back(g->words);
    delete g;
  });
}

pw_status future_new(pw_ctx* c, FutureRec** out, pw_future* handle) {
  uint32_t idx;
  if (!c->free_futures.empty()) {
    idx = c->free_futures.back();
    c->free_futures.pop_back();
  } else {
    idx = (uint32_t)c->futures.size();
    c->futures.emplace_back();
  }
  FutureRec& f = c->futures[idx];
  const uint32_t gen = f.gen + 1;
  f = FutureRec();
  f.gen = gen;
  f.live = true;
  f.refcount = 1;
  f.owner = c->current_owner;
  c->live_futures++;
  *out = &f;
  *handle = ((uint64_t)gen << 32) | (uint64_t)(idx + 1);
  return PW_OK;
}

FutureRec* future_get(pw_ctx* c, pw_future h) {
  const uint32_t idx = (uint32_t)(h & 0xFFFFFFFFu), gen = (uint32_t)(h >> 32);
  if (idx == 0 || idx > c->futures.size()) return nullptr;
  FutureRec& f = c->futures[idx - 1];
  return (f.live && f.gen == gen) ? &f : nullptr;
}

void future_drop(pw_ctx* c, pw_future h) {
  FutureRec* f = future_get(c, h);
  if (!f) return;
  if (--f->refcount > 0) return;
  if (f->gate) {
    // The gate kernel reads the flag word and the copy behind it reads the staging buffer: neither may be
    // recycled before they are done.  An unresolved gate is released first; the wait is then short.
    if (f->pending) __atomic_store_n(&f->gate->words[0], 2u, __ATOMIC_RELEASE);
    if (f->event) (void)hipEventSynchronize(f->event);
  }
  if (f->owns && f->buf) pool_free(c, f->buf, f->pool_bytes);
  if (f->event) c->event_pool.push_back(f->event);
  if (f->staging) c->staging_pool[size_class(f->bytes)].push_back(f->staging);
  f->poison.clear();
  f->gate.reset();
  f->live = false;
  c->live_futures--;
  c->free_futures.push_back((uint32_t)(h & 0xFFFFFFFFu) - 1);
}

FnRec* fn_get(pw_ctx* c, pw_fn h) {
  const uint32_t idx = (uint32_t)(h & 0xFFFFFFFFu), gen = (uint32_t)(h >> 32);
  if (idx == 0 || idx > c->fns.size()) return nullptr;
  FnRec& f = c->fns[idx - 1];
  return (f.live && f.gen == gen) ? &f : nullptr;
}

bool is_scalar_kind(int k) { return k >= PW_FN_ADD_CONST && k <= PW_FN_BUSY_CHAIN; }   // one fp32 input, one output

// Launch the body of one function on the executor stream.  in/out are device pointers.
pw_status fn_launch(pw_ctx* c, FnRec* fn, void* const* in, void* const* out) {
  const int k = fn->desc.kind;
  if (is_scalar_kind(k)) {
    hipError_t e = launch_scalar_fn(c->exec, k, (const float*)in[0], (float*)out[0], spec_numel(fn->desc.in[0]), fn->cst, fn->busy_us, fn->reps);
    if (e != hipSuccess) return fail(c, PW_ERR_DEVICE, "scalar fn launch: %s", hipGetErrorString(e));
    return PW_OK;
  }
  if (k == PW_FN_ADD2) {
    hipError_t e = launch_add2(c->exec, (const float*)in[0], (const float*)in[1], (float*)out[0], spec_numel(fn->desc.in[0]));
    if (e != hipSuccess) return fail(c, PW_ERR_DEVICE, "add2 launch: %s", hipGetErrorString(e));
    return PW_OK;
  }
  if (k == PW_FN_ENCDEC_TRAIN_STEP) {
    hipError_t e = encdec_train_step(fn->encdec, (const int32_t*)in[0], (const int32_t*)in[1], (float*)out[0]);
    if (e != hipSuccess) return fail(c, PW_ERR_DEVICE, "%s", fn->encdec->error.c_str());
    return PW_OK;
  }
  hipError_t e = hipErrorInvalidValue;
  if (k == PW_FN_LM_TRAIN_STEP) e = model_train_step(fn->model, (const int32_t*)in[0], (float*)out[0]);
  if (k == PW_FN_STAGE_FWD) e = model_stage_fwd(fn->model, fn->microbatch, (const float*)in[0], (float*)out[0]);
  if (k == PW_FN_STAGE_BWD) e = model_stage_bwd(fn->model, fn->microbatch, (const float*)in[0], (float*)out[0]);
  if (e != hipSuccess) return fail(c, PW_ERR_DEVICE, "%s", fn->model ? fn->model->error.c_str() : "bad function kind");
  return PW_OK;
}

// Checks n_in/n_out and every input spec against the compiled signature.
pw_status check_inputs(pw_ctx* c, FnRec* fn, const pw_tensor_spec* specs, int n_in, int n_out) {
  if (n_in != fn->desc.n_in || n_out != fn->desc.n_out)
    return fail(c, PW_ERR_SHAPE, "function takes %d inputs / %d outputs, got %d / %d", fn->desc.n_in, fn->desc.n_out, n_in, n_out);
  for (int i = 0; i < n_in; ++i) {
    pw_status st = spec_match(specs[i], fn->desc.in[i]);
    if (st != PW_OK) return fail(c, st, "input %d does not match the compiled signature", i);
  }
  return PW_OK;
}

// Make the executor stream wait for inputs produced elsewhere; collect poison dependencies.
pw_status wait_inputs(pw_ctx* c, FutureRec* const* in, int n_in, std::vector<std::shared_ptr<GateWords>>& poison, bool& host_poison) {
  for (int i = 0; i < n_in; ++i) {
    if (in[i]->on_gate_stream && in[i]->event) PW_HIP(c, hipStreamWaitEvent(c->exec, in[i]->event, 0));
    for (auto& p : in[i]->poison) poison.push_back(p);
    host_poison = host_poison || in[i]->host_poison;
  }
  return PW_OK;
}

bool model_alive(pw_ctx* c, Model* m) {
  for (Model* x : c->models)
    if (x == m) return true;
  return false;
}
bool encdec_alive(pw_ctx* c, EncDec* m) {
  for (EncDec* x : c->encdecs)
    if (x == m) return true;
  return false;
}

// ---- executors of pw_pipeline -------------------------------------------------------------------------
// HIP only orders a stream behind an event that has ALREADY been recorded, so a node's thread may not
// enqueue its wait before the producer's thread has recorded; that much of the order is kept on the host
// (wait_flag), everything else a thread does for its node runs concurrently with the other threads.
void executor_handle(int device, Executor* ex, NodeMsg& m) {
  bool ok = true;
  if (m.prep_us > 0) {   // host-side work for this node that needs nothing from its predecessor
    const auto t0 = std::chrono::steady_clock::now();
    while (std::chrono::steady_clock::now() - t0 < std::chrono::microseconds(m.prep_us)) {}
  }
  if (m.wait_flag) {
    const auto t0 = std::chrono::steady_clock::now();
    int v;
    while ((v = m.wait_flag->load(std::memory_order_acquire)) == 0) {
      if (std::chrono::steady_clock::now() - t0 > std::chrono::seconds(30)) { v = 2; break; }   // a thread that never reports: give up
      std::this_thread::yield();
    }
    ok = v == 1;
    if (ok && m.wait_event) ok = hipStreamWaitEvent(ex->stream, m.wait_event, 0) == hipSuccess;
  }
  if (ok) ok = launch_scalar_fn(ex->stream, m.kind, m.in, m.out, m.numel, m.cst, m.busy_us, m.reps) == hipSuccess;
  // "the source writes directly into the buffer the destination allocated" (Section 4.5)
  if (ok && m.xfer_dst && m.xfer_bytes) ok = launch_copy_bytes(ex->stream, m.out, m.xfer_dst, (int64_t)m.xfer_bytes) == hipSuccess;
  if (ok && m.done_event) ok = hipEventRecord(m.done_event, ex->stream) == hipSuccess;
  if (m.done_flag) m.done_flag->store(ok ? 1 : 2, std::memory_order_release);   // always: a consumer may be waiting
  m.ack->store(ok ? 1 : 2, std::memory_order_release);
  (void)device;
}

void executor_loop(int device, Executor* ex) {
  (void)hipSetDevice(device);
  for (;;) {
    NodeMsg m;
    {
      std::unique_lock<std::mutex> lk(ex->mu);
      ex->cv.wait(lk, [&] { return ex->stop || !ex->queue.empty(); });
      if (ex->queue.empty()) return;   // stop requested and nothing left
      m = ex->queue.front();
      ex->queue.pop_front();
    }
    executor_handle(device, ex, m);
  }
}

void stop_executors(pw_ctx* c) {
  for (auto& ex : c->executors) {
    {
      std::lock_guard<std::mutex> lk(ex->mu);
      ex->stop = true;
    }
    ex->cv.notify_all();
  }
  for (auto& ex : c->executors) {
    if (ex->thread.joinable()) ex->thread.join();
    if (ex->stream) (void)hipStreamSynchronize(ex->stream);
    if (ex->own_stream && ex->stream) (void)hipStreamDestroy(ex->stream);
  }
  c->executors.clear();
}

}  // namespace

// =====================================================================================================
extern "C" {

pw_status pw_ctx_create(int device, void* hip_stream, pw_ctx** out) {
  if (!out) return PW_ERR_INVALID;
  *out = nullptr;
  int n = 0;
  if (hipGetDeviceCount(&n) != hipSuccess || n <= 0 || device < 0 || device >= n) return PW_ERR_DEVICE;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device) != hipSuccess) return PW_ERR_DEVICE;
  if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return PW_ERR_UNSUPPORTED;   // kernels are built for gfx950 only
  if (hipSetDevice(device) != hipSuccess) return PW_ERR_DEVICE;
  pw_ctx* c = new pw_ctx();
  c->device = device;
  if (hip_stream) {
    c->exec = (hipStream_t)hip_stream;
  } else {
    if (hipStreamCreateWithFlags(&c->exec, hipStreamNonBlocking) != hipSuccess) { delete c; return PW_ERR_DEVICE; }
    c->own_exec = true;
  }
  if (hipStreamCreateWithFlags(&c->gate, hipStreamNonBlocking) != hipSuccess ||
      hipStreamCreateWithFlags(&c->io, hipStreamNonBlocking) != hipSuccess) {
    delete c;
    return PW_ERR_DEVICE;
  }
  if (gemm_init() != hipSuccess || attention_dma_init() != hipSuccess) {
    (void)hipStreamDestroy(c->gate);
    (void)hipStreamDestroy(c->io);
    if (c->own_exec) (void)hipStreamDestroy(c->exec);
    delete c;
    return PW_ERR_DEVICE;
  }
  *out = c;
  return PW_OK;
}

pw_status pw_ctx_destroy(pw_ctx* c) {
  if (!c) return PW_ERR_INVALID;
  (void)hipSetDevice(c->device);
  while (!c->scheds.empty()) (void)pw_sched_destroy(c->scheds.back());
  while (!c->programs.empty()) (void)pw_program_destroy(c->programs.back());
  stop_executors(c);
  // release every gate that is still waiting so that the streams can drain
  for (auto& f : c->futures)
    if (f.live && f.pending && f.gate) __atomic_store_n(&f.gate->words[0], 2u, __ATOMIC_RELEASE);
  (void)hipStreamSynchronize(c->gate);
  (void)hipStreamSynchronize(c->exec);
  (void)hipStreamSynchronize(c->io);
  for (auto& kv : c->graphs) {
    if (kv.second.exec) (void)hipGraphExecDestroy(kv.second.exec);
    if (kv.second.graph) (void)hipGraphDestroy(kv.second.graph);
  }
  for (Model* m : c->models) model_destroy(m);
  for (EncDec* m : c->encdecs) encdec_destroy(m);
  for (auto& f : c->futures) {
    if (!f.live) continue;
    if (f.owns && f.buf) (void)hipFree(f.buf);
    if (f.event) (void)hipEventDestroy(f.event);
    if (f.staging) (void)hipHostFree(f.staging);
    f.poison.clear();
    f.gate.reset();
  }
  for (auto& kv : c->pool)
    for (void* p : kv.second) (void)hipFree(p);
  for (auto& kv : c->staging_pool)
    for (void* p : kv.second) (void)hipHostFree(p);
  for (hipEvent_t e : c->event_pool) (void)hipEventDestroy(e);
  c->futures.clear();
  for (uint32_t* s : c->word_slabs) (void)hipHostFree(s);
  (void)hipStreamDestroy(c->gate);
  (void)hipStreamDestroy(c->io);
  if (c->own_exec) (void)hipStreamDestroy(c->exec);
  delete c;
  return PW_OK;
}

const char* pw_last_error(pw_ctx* c) { return c ? c->error.c_str() : "null context"; }
void* pw_ctx_stream(pw_ctx* c) { return c ? (void*)c->exec : nullptr; }

pw_status pw_ctx_synchronize(pw_ctx* c) {
  PW_API_LOCK(c);
  if (!c) return PW_ERR_INVALID;
  PW_HIP(c, hipStreamSynchronize(c->exec));
  return PW_OK;
}

pw_status pw_ctx_set_gate_timeout_ms(pw_ctx* c, int ms) {
  PW_API_LOCK(c);
  if (!c || ms < 1 || ms > 600000) return PW_ERR_INVALID;
  c->gate_timeout_ms = ms;
  return PW_OK;
}

pw_status pw_ctx_set_owner(pw_ctx* c, uint64_t owner) {
  PW_API_LOCK(c);
  if (!c) return PW_ERR_INVALID;
  c->current_owner = owner;
  return PW_OK;
}

pw_status pw_owner_collect(pw_ctx* c, uint64_t owner, int64_t* released) {
  PW_API_LOCK(c);
  if (!c) return PW_ERR_INVALID;
  int64_t n = 0;
  for (size_t i = 0; i < c->futures.size(); ++i) {
    FutureRec& f = c->futures[i];
    if (!f.live || f.owner != owner) continue;
    const pw_future h = ((uint64_t)f.gen << 32) | (uint64_t)(i + 1);
    if (f.on_gate_stream && f.event) {   // as in pw_future_release: the gate stream may still write the buffer
      if (f.pending) __atomic_store_n(&f.gate->words[0], 2u, __ATOMIC_RELEASE);
      (void)hipStreamWaitEvent(c->exec, f.event, 0);
    }
    f.refcount = 1;                      // every reference dies with the owner
    future_drop(c, h);
    ++n;
  }
  if (released) *released = n;
  return PW_OK;
}

pw_status pw_ctx_set_memory_limit(pw_ctx* c, int64_t bytes) {
  PW_API_LOCK(c);
  if (!c || bytes < 0) return PW_ERR_INVALID;
  c->memory_limit = bytes;
  return PW_OK;
}

pw_status pw_ctx_stats(pw_ctx* c, int64_t* live_futures, int64_t* pool_bytes_in_use) {
  PW_API_LOCK(c);
  if (!c) return PW_ERR_INVALID;
  if (live_futures) *live_futures = c->live_futures;
  if (pool_bytes_in_use) *pool_bytes_in_use = c->pool_in_use;
  return PW_OK;
}

// ---- compiled functions -----------------------------------------------------------------------------

pw_status pw_compile_fn(pw_ctx* c, const pw_fn_desc* d, pw_fn* out) {
  PW_API_LOCK(c);
  if (!c || !d || !out) return PW_ERR_INVALID;
  if (d->n_in < 0 || d->n_in > 8 || d->n_out < 0 || d->n_out > 8) return fail(c, PW_ERR_INVALID, "n_in / n_out out of range");
  for (int i = 0; i < d->n_in; ++i)
    if (!spec_ok(d->in[i])) return fail(c, PW_ERR_INVALID, "input spec %d is malformed", i);
  for (int i = 0; i < d->n_out; ++i)
    if (!spec_ok(d->out[i])) return fail(c, PW_ERR_INVALID, "output spec %d is malformed", i);
  FnRec fn;
  fn.desc = *d;
  fn.desc.params = nullptr;
  const int k = d->kind;
  if (is_scalar_kind(k)) {
    if (d->n_in != 1 || d->n_out != 1) return fail(c, PW_ERR_SHAPE, "elementwise functions take one input and give one output");
    if (d->in[0].dtype != PW_F32 || d->out[0].dtype != PW_F32) return fail(c, PW_ERR_DTYPE, "elementwise functions are fp32");
    pw_status st = spec_match(d->in[0], d->out[0]);
    if (st != PW_OK) return fail(c, st, "output must have the input's shape");
    const size_t need = (k == PW_FN_BUSY ? 2 : k == PW_FN_BUSY_CHAIN ? 3 : 1) * sizeof(float);
    if (!d->params || d->params_bytes != need) return fail(c, PW_ERR_INVALID, "params must hold %zu bytes", need);
    fn.cst = ((const float*)d->params)[0];
    if (k == PW_FN_BUSY || k == PW_FN_BUSY_CHAIN) {
      fn.busy_us = ((const float*)d->params)[1];
      if (!(fn.busy_us >= 0.f && fn.busy_us <= 1e6f)) return fail(c, PW_ERR_INVALID, "busy time must be within [0, 1e6] microseconds");
    }
    if (k == PW_FN_BUSY_CHAIN) {
      const float r = ((const float*)d->params)[2];
      if (!(r >= 1.f && r <= 65536.f) || r != (float)(int)r) return fail(c, PW_ERR_INVALID, "repetition count must be an integer within [1, 65536]");
      fn.reps = (int)r;
      if ((double)fn.busy_us * fn.reps > 1e7) return fail(c, PW_ERR_INVALID, "busy time times repetitions must stay within 1e7 microseconds");
    }
  } else if (k == PW_FN_ADD2) {
    if (d->n_in != 2 || d->n_out != 1) return fail(c, PW_ERR_SHAPE, "add2 takes two inputs and gives one output");
    if (d->in[0].dtype != PW_F32 || d->in[1].dtype != PW_F32 || d->out[0].dtype != PW_F32) return fail(c, PW_ERR_DTYPE, "add2 is fp32");
    pw_status st = spec_match(d->in[0], d->in[1]);
    if (st == PW_OK) st = spec_match(d->in[0], d->out[0]);
    if (st != PW_OK) return fail(c, st, "add2: inputs and output must have one shape");
    if (d->params_bytes != 0) return fail(c, PW_ERR_INVALID, "add2 takes no params");
  } else if (k == PW_FN_LM_TRAIN_STEP || k == PW_FN_STAGE_FWD || k == PW_FN_STAGE_BWD) {
    pw_model* pm = nullptr;
    if (k == PW_FN_LM_TRAIN_STEP) {
      if (!d->params || d->params_bytes != sizeof(pw_model*)) return fail(c, PW_ERR_INVALID, "params must hold a pw_model*");
      std::memcpy(&pm, d->params, sizeof pm);
    } else {
      if (!d->params || d->params_bytes != sizeof(pw_stage_params)) return fail(c, PW_ERR_INVALID, "params must hold pw_stage_params");
      pw_stage_params sp;
      std::memcpy(&sp, d->params, sizeof sp);
      pm = sp.model;
      fn.microbatch = sp.microbatch;
    }
    if (!pm || pm->ctx != c || !model_alive(c, pm->impl)) return fail(c, PW_ERR_INVALID, "model does not belong to this context");
    fn.model = pm->impl;
    const pw_lm_config& cfg = fn.model->cfg;
    if (d->n_in != 1 || d->n_out != 1) return fail(c, PW_ERR_SHAPE, "one input and one output expected");
    pw_tensor_spec want_in{}, want_out{};
    if (k == PW_FN_LM_TRAIN_STEP) {
      if (!cfg.has_embed || !cfg.has_head) return fail(c, PW_ERR_UNSUPPORTED, "model is a pipeline stage, not a full LM");
      want_in = {PW_I32, 2, {cfg.batch, cfg.seq + 1, 0, 0}};
      want_out = {PW_F32, 1, {1, 0, 0, 0}};
    } else {
      if (cfg.has_embed || cfg.has_head) return fail(c, PW_ERR_UNSUPPORTED, "model is a full LM, not a pipeline stage");
      if (fn.microbatch < 0 || fn.microbatch >= cfg.n_microbatch) return fail(c, PW_ERR_INVALID, "micro-batch index out of range");
      want_in = {PW_F32, 2, {(int64_t)cfg.batch * cfg.seq, cfg.d_model, 0, 0}};
      want_out = want_in;
    }
    pw_status st = spec_match(d->in[0], want_in);
    if (st != PW_OK) return fail(c, st, "input signature does not fit the model");
    st = spec_match(d->out[0], want_out);
    if (st != PW_OK) return fail(c, st, "output signature does not fit the model");
  } else if (k == PW_FN_ENCDEC_TRAIN_STEP) {
    pw_encdec* pm = nullptr;
    if (!d->params || d->params_bytes != sizeof(pw_encdec*)) return fail(c, PW_ERR_INVALID, "params must hold a pw_encdec*");
    std::memcpy(&pm, d->params, sizeof pm);
    if (!pm || pm->ctx != c || !encdec_alive(c, pm->impl)) return fail(c, PW_ERR_INVALID, "model does not belong to this context");
    fn.encdec = pm->impl;
    const pw_encdec_config& cfg = fn.encdec->cfg;
    if (d->n_in != 2 || d->n_out != 1) return fail(c, PW_ERR_SHAPE, "two inputs (source, target tokens) and one output expected");
    const pw_tensor_spec want_src{PW_I32, 2, {cfg.batch, cfg.src_len, 0, 0}}, want_tgt{PW_I32, 2, {cfg.batch, cfg.tgt_len + 1, 0, 0}};
    const pw_tensor_spec want_out{PW_F32, 1, {1, 0, 0, 0}};
    pw_status st = spec_match(d->in[0], want_src);
    if (st == PW_OK) st = spec_match(d->in[1], want_tgt);
    if (st != PW_OK) return fail(c, st, "input signature does not fit the model");
    st = spec_match(d->out[0], want_out);
    if (st != PW_OK) return fail(c, st, "output signature does not fit the model");
  } else {
    return fail(c, PW_ERR_INVALID, "unknown function kind %d", k);
  }
  uint32_t idx = (uint32_t)c->fns.size();
  for (uint32_t i = 0; i < c->fns.size(); ++i)
    if (!c->fns[i].live) { idx = i; break; }
  if (idx == c->fns.size()) c->fns.emplace_back();
  const uint32_t gen = c->fns[idx].gen + 1;
  c->fns[idx] = fn;
  c->fns[idx].gen = gen;
  c->fns[idx].live = true;
  *out = ((uint64_t)gen << 32) | (uint64_t)(idx + 1);
  return PW_OK;
}

pw_status pw_fn_release(pw_ctx* c, pw_fn h) {
  PW_API_LOCK(c);
  if (!c) return PW_ERR_INVALID;
  FnRec* f = fn_get(c, h);
  if (!f) return fail(c, PW_ERR_INVALID, "bad function handle");
  f->live = false;
  return PW_OK;
}

pw_status pw_run_fn(pw_ctx* c, pw_fn h, const pw_future* in, int n_in, pw_future* out, int n_out) {
  PW_API_LOCK(c);
  if (!c || (n_in > 0 && !in) || (n_out > 0 && !out) || n_in < 0 || n_in > 8 || n_out < 0 || n_out > 8) return PW_ERR_INVALID;
  FnRec* fn = fn_get(c, h);
  if (!fn) return fail(c, PW_ERR_INVALID, "bad function handle");
  FutureRec* fin[8];
  pw_tensor_spec specs[8];
  for (int i = 0; i < n_in; ++i) {
    fin[i] = future_get(c, in[i]);
    if (!fin[i]) return fail(c, PW_ERR_INVALID, "input %d is not a live future", i);
    specs[i] = fin[i]->spec;
  }
  pw_status st = check_inputs(c, fn, specs, n_in, n_out);
  if (st != PW_OK) return st;
  // everything is validated: from here on we enqueue
  void* obuf[8];
  size_t ocls[8];
  for (int i = 0; i < n_out; ++i) {
    st = pool_alloc(c, spec_bytes(fn->desc.out[i]), &obuf[i], &ocls[i]);
    if (st != PW_OK) {
      for (int j = 0; j < i; ++j) pool_free(c, obuf[j], ocls[j]);
      return st;
    }
  }
  std::vector<std::shared_ptr<GateWords>> poison;
  bool host_poison = false;
  st = wait_inputs(c, fin, n_in, poison, host_poison);
  void* ibuf[8];
  for (int i = 0; i < n_in; ++i) ibuf[i] = fin[i]->buf;
  if (st == PW_OK) st = fn_launch(c, fn, ibuf, obuf);
  hipEvent_t ev = nullptr;
  if (st == PW_OK) st = event_get(c, &ev);
  if (st == PW_OK && hipEventRecord(ev, c->exec) != hipSuccess) st = fail(c, PW_ERR_DEVICE, "hipEventRecord failed");
  if (st != PW_OK) {
    for (int i = 0; i < n_out; ++i) pool_free(c, obuf[i], ocls[i]);
    if (ev) c->event_pool.push_back(ev);
    return st;
  }
  for (int i = 0; i < n_out; ++i) {
    FutureRec* f;
    future_new(c, &f, &out[i]);
    // the vector may have grown: input records are not touched below
    f->buf = obuf[i];
    f->bytes = spec_bytes(fn->desc.out[i]);
    f->pool_bytes = ocls[i];
    f->spec = fn->desc.out[i];
    f->owns = true;
    f->poison = poison;
    f->host_poison = host_poison;
    if (i == 0) {
      f->event = ev;
    } else {   // one event per future keeps release simple
      hipEvent_t e2;
      if (event_get(c, &e2) == PW_OK && hipEventRecord(e2, c->exec) == hipSuccess) f->event = e2;
    }
  }
  return PW_OK;
}

pw_status pw_chain(pw_ctx* c, const pw_fn* fns, int n_fns, const pw_future* in, int n_in, pw_future* out, int n_out, int mode) {
  PW_API_LOCK(c);
  if (!c || !fns || n_fns < 1 || n_fns > 4096 || (n_in > 0 && !in) || (n_out > 0 && !out) || n_in < 0 || n_in > 8 || n_out < 0 || n_out > 8)
    return PW_ERR_INVALID;
  if (mode != PW_STREAM && mode != PW_GRAPH && mode != PW_SEQUENTIAL) return fail(c, PW_ERR_INVALID, "bad chain mode");
  // ---- validate the whole chain before touching the device
  std::vector<FnRec*> recs(n_fns);
  for (int i = 0; i < n_fns; ++i) {
    recs[i] = fn_get(c, fns[i]);
    if (!recs[i]) return fail(c, PW_ERR_INVALID, "function %d of the chain is not a live handle", i);
  }
  FutureRec* fin[8];
  pw_tensor_spec specs[8];
  for (int i = 0; i < n_in; ++i) {
    fin[i] = future_get(c, in[i]);
    if (!fin[i]) return fail(c, PW_ERR_INVALID, "input %d is not a live future", i);
    specs[i] = fin[i]->spec;
  }
  int cur_n = n_in;
  for (int i = 0; i < n_fns; ++i) {
    const int want_out = i + 1 < n_fns ? recs[i]->desc.n_out : n_out;
    pw_status st = check_inputs(c, recs[i], specs, cur_n, want_out);
    if (st != PW_OK) {
      c->error = "chain link " + std::to_string(i) + ": " + c->error;
      return st;
    }
    cur_n = recs[i]->desc.n_out;
    for (int j = 0; j < cur_n; ++j) specs[j] = recs[i]->desc.out[j];
  }
  // ---- allocate every buffer the chain needs (two alternating sets of intermediates, then the outputs)
  struct Buf { void* p; size_t cls; };
  std::vector<std::vector<Buf>> bufs(n_fns);
  auto release_all = [&]() {
    for (auto& v : bufs)
      for (auto& b : v) pool_free(c, b.p, b.cls);
  };
  // Intermediates of link i can be recycled once link i+1 has been enqueued; allocating and freeing in
  // that order makes the pool hand back the same few buffers, so the address pattern repeats call after
  // call (which is what lets a cached graph be replayed unchanged).
  std::vector<std::vector<Buf>> plan_bufs(n_fns);
  {
    std::vector<Buf> prev;
    for (int i = 0; i < n_fns; ++i) {
      for (int j = 0; j < recs[i]->desc.n_out; ++j) {
        Buf b;
        pw_status st = pool_alloc(c, spec_bytes(recs[i]->desc.out[j]), &b.p, &b.cls);
        if (st != PW_OK) {
          for (auto& x : prev) pool_free(c, x.p, x.cls);
          for (auto& x : plan_bufs[i]) pool_free(c, x.p, x.cls);
          return st;
        }
        plan_bufs[i].push_back(b);
      }
      for (auto& x : prev) pool_free(c, x.p, x.cls);   // stream order keeps reuse safe
      prev = plan_bufs[i];
    }
    bufs[n_fns - 1] = prev;   // only the last link's buffers stay allocated
  }
  std::vector<std::shared_ptr<GateWords>> poison;
  bool host_poison = false;
  pw_status st = wait_inputs(c, fin, n_in, poison, host_poison);
  if (st != PW_OK) { release_all(); return st; }

  auto enqueue_all = [&](bool sync_each) -> pw_status {
    void* ibuf[8];
    void* obuf[8];
    for (int j = 0; j < n_in; ++j) ibuf[j] = fin[j]->buf;
    for (int i = 0; i < n_fns; ++i) {
      for (size_t j = 0; j < plan_bufs[i].size(); ++j) obuf[j] = plan_bufs[i][j].p;
      pw_status s2 = fn_launch(c, recs[i], ibuf, obuf);
      if (s2 != PW_OK) return s2;
      if (sync_each && hipStreamSynchronize(c->exec) != hipSuccess) return fail(c, PW_ERR_DEVICE, "stream synchronize failed");
      for (size_t j = 0; j < plan_bufs[i].size(); ++j) ibuf[j] = obuf[j];
    }
    return PW_OK;
  };

  if (mode == PW_GRAPH) {
    std::string key;
    key.append((const char*)fns, sizeof(pw_fn) * n_fns);
    for (int j = 0; j < n_in; ++j) key.append((const char*)&fin[j]->buf, sizeof(void*));
    for (auto& v : plan_bufs)
      for (auto& b : v) key.append((const char*)&b.p, sizeof(void*));
    auto it = c->graphs.find(key);
    if (it == c->graphs.end()) {
      if (c->graphs.size() >= 256) {   // bounded cache: drop everything rather than grow without limit
        for (auto& kv : c->graphs) {
          (void)hipGraphExecDestroy(kv.second.exec);
          (void)hipGraphDestroy(kv.second.graph);
        }
        c->graphs.clear();
      }
      GraphEntry ge;
      hipError_t e = hipStreamBeginCapture(c->exec, hipStreamCaptureModeThreadLocal);
      if (e != hipSuccess) { release_all(); return fail(c, PW_ERR_DEVICE, "begin capture: %s", hipGetErrorString(e)); }
      st = enqueue_all(false);
      e = hipStreamEndCapture(c->exec, &ge.graph);
      if (st != PW_OK || e != hipSuccess || !ge.graph) {
        if (ge.graph) (void)hipGraphDestroy(ge.graph);
        release_all();
        return st != PW_OK ? st : fail(c, PW_ERR_DEVICE, "end capture: %s", hipGetErrorString(e));
      }
      e = hipGraphInstantiate(&ge.exec, ge.graph, nullptr, nullptr, 0);
      if (e != hipSuccess) {
        (void)hipGraphDestroy(ge.graph);
        release_all();
        return fail(c, PW_ERR_DEVICE, "graph instantiate: %s", hipGetErrorString(e));
      }
      it = c->graphs.emplace(key, ge).first;
    }
    hipError_t e = hipGraphLaunch(it->second.exec, c->exec);
    if (e != hipSuccess) { release_all(); return fail(c, PW_ERR_DEVICE, "graph launch: %s", hipGetErrorString(e)); }
  } else {
    st = enqueue_all(mode == PW_SEQUENTIAL);
    if (st != PW_OK) { release_all(); return st; }
  }
  hipEvent_t ev = nullptr;
  st = event_get(c, &ev);
  if (st == PW_OK && hipEventRecord(ev, c->exec) != hipSuccess) st = fail(c, PW_ERR_DEVICE, "hipEventRecord failed");
  if (st != PW_OK) { release_all(); return st; }
  for (int i = 0; i < n_out; ++i) {
    FutureRec* f;
    future_new(c, &f, &out[i]);
    f->buf = bufs[n_fns - 1][i].p;
    f->pool_bytes = bufs[n_fns - 1][i].cls;
    f->spec = recs[n_fns - 1]->desc.out[i];
    f->bytes = spec_bytes(f->spec);
    f->owns = true;
    f->poison = poison;
    f->host_poison = host_poison;
    if (i == 0) {
      f->event = ev;
    } else {
      hipEvent_t e2;
      if (event_get(c, &e2) == PW_OK && hipEventRecord(e2, c->exec) == hipSuccess) f->event = e2;
    }
  }
  return PW_OK;
}

pw_status pw_ctx_set_executors(pw_ctx* c, int n) {
  PW_API_LOCK(c);
  if (!c) return PW_ERR_INVALID;
  if (n < 1 || n > 64) return fail(c, PW_ERR_INVALID, "executor count must be within [1, 64]");
  if (!c->executors.empty()) return fail(c, PW_ERR_INVALID, "executors are already set up");
  (void)hipSetDevice(c->device);
  for (int i = 0; i < n; ++i) {
    std::unique_ptr<Executor> ex(new Executor());
    if (i == 0) {
      ex->stream = c->exec;
    } else {
      if (hipStreamCreateWithFlags(&ex->stream, hipStreamNonBlocking) != hipSuccess) {
        stop_executors(c);
        return fail(c, PW_ERR_DEVICE, "could not create the stream of executor %d", i);
      }
      ex->own_stream = true;
    }
    c->executors.push_back(std::move(ex));
  }
  for (auto& ex : c->executors) ex->thread = std::thread(executor_loop, c->device, ex.get());
  return PW_OK;
}

pw_status pw_ctx_set_executor_prep_us(pw_ctx* c, int us) {
  PW_API_LOCK(c);
  if (!c || us < 0 || us > 100000) return PW_ERR_INVALID;
  c->executor_prep_us = us;
  return PW_OK;
}

pw_status pw_pipeline(pw_ctx* c, const pw_fn* fns, const int32_t* executor_of, int n_fns, pw_future in, pw_future* out, int dispatch) {
  PW_API_LOCK(c);
  if (!c || !fns || !executor_of || !out || n_fns < 1 || n_fns > 4096) return PW_ERR_INVALID;
  if (dispatch != PW_DISPATCH_PARALLEL && dispatch != PW_DISPATCH_SEQUENTIAL) return fail(c, PW_ERR_INVALID, "bad dispatch mode");
  if (c->executors.empty()) return fail(c, PW_ERR_INVALID, "call pw_ctx_set_executors first");
  // ---- validate everything before touching the device
  std::vector<FnRec*> recs(n_fns);
  FutureRec* fin = future_get(c, in);
  if (!fin) return fail(c, PW_ERR_INVALID, "input is not a live future");
  pw_tensor_spec spec = fin->spec;
  for (int i = 0; i < n_fns; ++i) {
    recs[i] = fn_get(c, fns[i]);
    if (!recs[i]) return fail(c, PW_ERR_INVALID, "function %d of the pipeline is not a live handle", i);
    if (!is_scalar_kind(recs[i]->desc.kind)) return fail(c, PW_ERR_UNSUPPORTED, "node %d: only elementwise functions can be placed on an executor", i);
    if (executor_of[i] < 0 || executor_of[i] >= (int)c->executors.size()) return fail(c, PW_ERR_INVALID, "node %d: no executor %d", i, executor_of[i]);
    pw_status st = check_inputs(c, recs[i], &spec, 1, 1);
    if (st != PW_OK) {
      c->error = "pipeline node " + std::to_string(i) + ": " + c->error;
      return st;
    }
    spec = recs[i]->desc.out[0];
  }
  const size_t bytes = spec_bytes(spec);   // elementwise: every node has the input's shape
  // ---- plan: per node an output buffer, and where it crosses executors a consumer-side input buffer + event
  struct Plan { void* out = nullptr; size_t out_cls = 0; void* xfer = nullptr; size_t xfer_cls = 0; hipEvent_t ev = nullptr; };
  std::vector<Plan> plan(n_fns);
  auto release_plan = [&](bool keep_last) {
    for (int i = 0; i < n_fns; ++i) {
      if (plan[i].out && !(keep_last && i == n_fns - 1)) pool_free(c, plan[i].out, plan[i].out_cls);
      if (plan[i].xfer) pool_free(c, plan[i].xfer, plan[i].xfer_cls);
      if (plan[i].ev && !(keep_last && i == n_fns - 1)) c->event_pool.push_back(plan[i].ev);
    }
  };
  for (int i = 0; i < n_fns; ++i) {
    pw_status st = pool_alloc(c, bytes, &plan[i].out, &plan[i].out_cls);
    const bool crosses = i + 1 < n_fns && executor_of[i + 1] != executor_of[i];
    if (st == PW_OK && crosses) st = pool_alloc(c, bytes, &plan[i].xfer, &plan[i].xfer_cls);
    if (st == PW_OK && (crosses || i == n_fns - 1)) st = event_get(c, &plan[i].ev);
    if (st != PW_OK) { release_plan(false); return st; }
  }
  // the first node's stream must be ordered behind the producer of `in` (and behind earlier users of the pool's
  // buffers, which all ran on streams this context has since been synchronised with or on the executor stream)
  std::vector<std::shared_ptr<GateWords>> poison = fin->poison;
  bool host_poison = fin->host_poison;
  hipEvent_t order = nullptr;
  pw_status st = event_get(c, &order);
  if (st != PW_OK) { release_plan(false); return st; }
  hipError_t e = hipSuccess;
  if (fin->on_gate_stream && fin->event) e = hipStreamWaitEvent(c->exec, fin->event, 0);
  if (e == hipSuccess) e = hipEventRecord(order, c->exec);
  std::vector<char> used(c->executors.size(), 0);
  for (int i = 0; i < n_fns; ++i) used[executor_of[i]] = 1;
  for (size_t x = 1; x < c->executors.size() && e == hipSuccess; ++x)
    if (used[x]) e = hipStreamWaitEvent(c->executors[x]->stream, order, 0);
  c->event_pool.push_back(order);
  if (e != hipSuccess) { release_plan(false); return fail(c, PW_ERR_DEVICE, "ordering the executors: %s", hipGetErrorString(e)); }

  // ---- dispatch
  std::vector<std::atomic<int>> acks(n_fns), flags(n_fns);
  for (int i = 0; i < n_fns; ++i) { acks[i].store(0); flags[i].store(0); }
  auto post = [&](int i) {
    NodeMsg m;
    m.kind = recs[i]->desc.kind; m.cst = recs[i]->cst; m.busy_us = recs[i]->busy_us; m.reps = recs[i]->reps;
    m.numel = spec_numel(spec);
    const bool from_other = i > 0 && executor_of[i - 1] != executor_of[i];
    m.in = (const float*)(i == 0 ? fin->buf : from_other ? plan[i - 1].xfer : plan[i - 1].out);
    m.out = (float*)plan[i].out;
    m.xfer_dst = plan[i].xfer; m.xfer_bytes = plan[i].xfer ? bytes : 0;
    if (from_other) { m.wait_event = plan[i - 1].ev; m.wait_flag = &flags[i - 1]; }
    else if (i > 0) { m.wait_flag = &flags[i - 1]; }   // same stream: only the host-side order of the two enqueues matters
    m.done_event = plan[i].ev; m.done_flag = &flags[i]; m.ack = &acks[i];
    m.prep_us = c->executor_prep_us;
    Executor* ex = c->executors[executor_of[i]].get();
    {
      std::lock_guard<std::mutex> lk(ex->mu);
      ex->queue.push_back(m);
    }
    ex->cv.notify_one();
  };
  auto wait_ack = [&](int i) {
    while (acks[i].load(std::memory_order_acquire) == 0) std::this_thread::yield();
    return acks[i].load(std::memory_order_acquire) == 1;
  };
  bool all_ok = true;
  if (dispatch == PW_DISPATCH_PARALLEL) {
    for (int i = 0; i < n_fns; ++i) post(i);                      // every node's host-side work starts now
    for (int i = 0; i < n_fns; ++i) all_ok = wait_ack(i) && all_ok;
  } else {
    for (int i = 0; i < n_fns; ++i) {                             // node i+1 is handed out once node i reports "enqueued"
      post(i);
      all_ok = wait_ack(i) && all_ok;
    }
  }
  // Intermediates go back to the pool: their last use is already enqueued; later users are ordered behind the
  // executor stream, which is made to wait for the last node below.
  FutureRec* f;
  future_new(c, &f, out);
  f->buf = plan[n_fns - 1].out; f->pool_bytes = plan[n_fns - 1].out_cls; f->spec = spec; f->bytes = bytes; f->owns = true;
  f->poison = poison;
  f->host_poison = host_poison || !all_ok;
  f->event = plan[n_fns - 1].ev;
  // join: everything enqueued on the executor stream from now on runs after the whole pipeline
  for (size_t x = 1; x < c->executors.size(); ++x) {
    hipEvent_t j = nullptr;
    if (used[x] && event_get(c, &j) == PW_OK) {
      if (hipEventRecord(j, c->executors[x]->stream) == hipSuccess) (void)hipStreamWaitEvent(c->exec, j, 0);
      c->event_pool.push_back(j);
    }
  }
  release_plan(true);
  if (!all_ok) return fail(c, PW_ERR_DEVICE, "a pipeline node could not be enqueued; the output future is poisoned");
  return PW_OK;
}

// ---- dataflow programs ---------------------------------------------------------------------------------------
pw_status pw_program_create(pw_ctx* c, const pw_tensor_spec* input_specs, int n_inputs, const pw_node* nodes, int n_nodes,
                            const int32_t* outputs, int n_outputs, pw_program** out) {
  if (!c || !out || !nodes || !outputs || (n_inputs > 0 && !input_specs)) return PW_ERR_INVALID;
  PW_API_LOCK(c);
  if (n_inputs < 0 || n_inputs > 8 || n_nodes < 1 || n_nodes > 4096 || n_outputs < 1 || n_outputs > 8)
    return fail(c, PW_ERR_INVALID, "a program has 0..8 inputs, 1..4096 nodes and 1..8 outputs");
  std::unique_ptr<pw_program> p(new pw_program());
  p->ctx = c;
  p->n_inputs = n_inputs;
  for (int i = 0; i < n_inputs; ++i) {
    if (!spec_ok(input_specs[i])) return fail(c, PW_ERR_INVALID, "input spec %d is malformed", i);
    p->specs.push_back(input_specs[i]);
  }
  for (int i = 0; i < n_nodes; ++i) {
    FnRec* fn = fn_get(c, nodes[i].fn);
    if (!fn) return fail(c, PW_ERR_INVALID, "node %d: not a live function handle", i);
    if (nodes[i].n_in != fn->desc.n_in) return fail(c, PW_ERR_SHAPE, "node %d: function takes %d inputs, the trace gives %d", i, fn->desc.n_in, nodes[i].n_in);
    ProgNode n;
    n.fn = *fn;
    n.handle = nodes[i].fn;
    n.n_in = nodes[i].n_in;
    for (int j = 0; j < n.n_in; ++j) {
      const int v = nodes[i].in[j];
      if (v < 0 || v >= (int)p->specs.size()) return fail(c, PW_ERR_INVALID, "node %d: input %d names value %d, which is not defined before it", i, j, v);
      pw_status st = spec_match(p->specs[v], fn->desc.in[j]);
      if (st != PW_OK) return fail(c, st, "node %d: value %d does not match input %d of the compiled signature", i, v, j);
      n.in[j] = v;
    }
    n.first_out = (int)p->specs.size();
    for (int j = 0; j < fn->desc.n_out; ++j) p->specs.push_back(fn->desc.out[j]);
    p->nodes.push_back(n);
  }
  p->last_use.assign(p->specs.size(), -1);
  for (int i = 0; i < n_nodes; ++i)
    for (int j = 0; j < p->nodes[i].n_in; ++j) p->last_use[p->nodes[i].in[j]] = i;
  for (int i = 0; i < n_outputs; ++i) {
    const int v = outputs[i];
    if (v < 0 || v >= (int)p->specs.size()) return fail(c, PW_ERR_INVALID, "output %d names value %d, which does not exist", i, v);
    if (v < n_inputs) return fail(c, PW_ERR_UNSUPPORTED, "output %d is a program input; return it from the caller instead", i);
    for (int k = 0; k < i; ++k)
      if (outputs[k] == v) return fail(c, PW_ERR_UNSUPPORTED, "value %d is returned twice", v);
    p->last_use[v] = n_nodes;
    p->outputs.push_back(v);
  }
  c->programs.push_back(p.get());
  *out = p.release();
  return PW_OK;
}

pw_status pw_program_destroy(pw_program* p) {
  if (!p) return PW_ERR_INVALID;
  pw_ctx* c = p->ctx;
  PW_API_LOCK(c);
  (void)hipStreamSynchronize(c->exec);   // a replay may still be running
  for (auto& kv : p->graphs) {
    if (kv.second.exec) (void)hipGraphExecDestroy(kv.second.exec);
    if (kv.second.graph) (void)hipGraphDestroy(kv.second.graph);
  }
  for (size_t i = 0; i < c->programs.size(); ++i)
    if (c->programs[i] == p) { c->programs.erase(c->programs.begin() + i); break; }
  delete p;
  return PW_OK;
}

pw_status pw_program_run(pw_ctx* c, pw_program* p, const pw_future* in, int n_in, pw_future* out, int n_out, int mode) {
  if (!c || !p || p->ctx != c || (n_in > 0 && !in) || !out) return PW_ERR_INVALID;
  PW_API_LOCK(c);
  if (mode != PW_STREAM && mode != PW_GRAPH) return fail(c, PW_ERR_INVALID, "programs run in PW_STREAM or PW_GRAPH mode");
  if (n_in != p->n_inputs || n_out != (int)p->outputs.size())
    return fail(c, PW_ERR_SHAPE, "program takes %d inputs / gives %zu outputs, got %d / %d", p->n_inputs, p->outputs.size(), n_in, n_out);
  FutureRec* fin[8];
  for (int i = 0; i < n_in; ++i) {
    fin[i] = future_get(c, in[i]);
    if (!fin[i]) return fail(c, PW_ERR_INVALID, "input %d is not a live future", i);
    pw_status st = spec_match(fin[i]->spec, p->specs[i]);
    if (st != PW_OK) return fail(c, st, "input %d does not match the traced signature", i);
  }
  // ---- buffer plan: allocate each value when its producer is reached, give it back when its last consumer has
  // been passed (stream order keeps the reuse safe; the pool then repeats the same addresses call after call)
  const int n_nodes = (int)p->nodes.size();
  struct Buf { void* p = nullptr; size_t cls = 0; };
  std::vector<Buf> val(p->specs.size());
  for (int i = 0; i < n_in; ++i) val[i].p = fin[i]->buf;
  std::vector<char> held(p->specs.size(), 0);
  for (int i = 0; i < n_nodes; ++i) {
    const ProgNode& n = p->nodes[i];
    for (int j = 0; j < n.fn.desc.n_out; ++j) {
      const int v = n.first_out + j;
      pw_status st = pool_alloc(c, spec_bytes(p->specs[v]), &val[v].p, &val[v].cls);
      if (st != PW_OK) {
        for (size_t w = p->n_inputs; w < val.size(); ++w)
          if (held[w]) pool_free(c, val[w].p, val[w].cls);
        return st;
      }
      held[v] = 1;
    }
    for (int j = 0; j < n.n_in; ++j) {
      const int v = n.in[j];
      if (v >= p->n_inputs && held[v] && p->last_use[v] == i) { pool_free(c, val[v].p, val[v].cls); held[v] = 0; }
    }
    for (int j = 0; j < n.fn.desc.n_out; ++j) {   // produced but never read nor returned
      const int v = n.first_out + j;
      if (p->last_use[v] < 0) { pool_free(c, val[v].p, val[v].cls); held[v] = 0; }
    }
  }
  auto release_outputs = [&]() {
    for (int v : p->outputs)
      if (held[v]) { pool_free(c, val[v].p, val[v].cls); held[v] = 0; }
  };
  std::vector<std::shared_ptr<GateWords>> poison;
  bool host_poison = false;
  pw_status st = wait_inputs(c, fin, n_in, poison, host_poison);
  if (st != PW_OK) { release_outputs(); return st; }

  auto enqueue_all = [&]() -> pw_status {
    for (int i = 0; i < n_nodes; ++i) {
      ProgNode& n = p->nodes[i];
      void* ibuf[8];
      void* obuf[8];
      for (int j = 0; j < n.n_in; ++j) ibuf[j] = val[n.in[j]].p;
      for (int j = 0; j < n.fn.desc.n_out; ++j) obuf[j] = val[n.first_out + j].p;
      pw_status s2 = fn_launch(c, &n.fn, ibuf, obuf);
      if (s2 != PW_OK) return s2;
    }
    return PW_OK;
  };
  if (mode == PW_GRAPH) {
    std::string key;
    for (auto& b : val) key.append((const char*)&b.p, sizeof(void*));
    auto it = p->graphs.find(key);
    if (it == p->graphs.end()) {
      if (p->graphs.size() >= 64) {
        (void)hipStreamSynchronize(c->exec);
        for (auto& kv : p->graphs) {
          (void)hipGraphExecDestroy(kv.second.exec);
          (void)hipGraphDestroy(kv.second.graph);
        }
        p->graphs.clear();
      }
      GraphEntry ge;
      hipError_t e = hipStreamBeginCapture(c->exec, hipStreamCaptureModeThreadLocal);
      if (e != hipSuccess) { release_outputs(); return fail(c, PW_ERR_DEVICE, "begin capture: %s", hipGetErrorString(e)); }
      st = enqueue_all();
      e = hipStreamEndCapture(c->exec, &ge.graph);
      if (st != PW_OK || e != hipSuccess || !ge.graph) {
        if (ge.graph) (void)hipGraphDestroy(ge.graph);
        release_outputs();
        return st != PW_OK ? st : fail(c, PW_ERR_DEVICE, "end capture: %s", hipGetErrorString(e));
      }
      e = hipGraphInstantiate(&ge.exec, ge.graph, nullptr, nullptr, 0);
      if (e != hipSuccess) {
        (void)hipGraphDestroy(ge.graph);
        release_outputs();
        return fail(c, PW_ERR_DEVICE, "graph instantiate: %s", hipGetErrorString(e));
      }
      it = p->graphs.emplace(key, ge).first;
    }
    hipError_t e = hipGraphLaunch(it->second.exec, c->exec);
    if (e != hipSuccess) { release_outputs(); return fail(c, PW_ERR_DEVICE, "graph launch: %s", hipGetErrorString(e)); }
  } else {
    st = enqueue_all();
    if (st != PW_OK) { release_outputs(); return st; }
  }
  for (int i = 0; i < n_out; ++i) {
    const int v = p->outputs[i];
    hipEvent_t ev = nullptr;
    if (event_get(c, &ev) == PW_OK && hipEventRecord(ev, c->exec) != hipSuccess) { c->event_pool.push_back(ev); ev = nullptr; }
    FutureRec* f;
    future_new(c, &f, &out[i]);
    f->buf = val[v].p; f->pool_bytes = val[v].cls; f->spec = p->specs[v]; f->bytes = spec_bytes(f->spec); f->owns = true;
    f->poison = poison; f->host_poison = host_poison; f->event = ev;
  }
  return PW_OK;
}

// ---- scheduler ---------------------------------------------------------------------------------------------
namespace {

hipEvent_t sched_event(pw_sched* s) {
  if (!s->timing_events.empty()) {
    hipEvent_t e = s->timing_events.back();
    s->timing_events.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

// Retire the oldest program in flight: wait for it, charge its device time to its client.
void sched_retire(pw_sched* s) {
  SchedInFlight f = s->inflight.front();
  s->inflight.pop_front();
  float ms = 0.f, t0 = 0.f;
  const bool ok = f.start && f.stop && hipEventSynchronize(f.stop) == hipSuccess &&
                  hipEventElapsedTime(&ms, f.start, f.stop) == hipSuccess &&
                  hipEventElapsedTime(&t0, s->epoch, f.start) == hipSuccess;
  std::lock_guard<std::mutex> lk(s->mu);
  if (ok) {
    SchedClient& c = s->clients[f.client];
    c.device_ms += ms;
    if (s->trace.size() < 65536) s->trace.push_back(pw_sched_slice{f.client, f.n_computations, t0, t0 + ms});
  }
  if (f.start) s->timing_events.push_back(f.start);
  if (f.stop) s->timing_events.push_back(f.stop);
}

void sched_loop(pw_sched* s) {
  (void)hipSetDevice(s->ctx->device);
  for (;;) {
    SchedProgram prog;
    int client = -1;
    {
      std::unique_lock<std::mutex> lk(s->mu);
      while (!s->stop && s->queued == 0) {
        if (!s->inflight.empty()) {          // nothing to hand out: use the time to retire finished programs
          lk.unlock();
          sched_retire(s);
          lk.lock();
          continue;
        }
        s->idle = true;
        s->cv_done.notify_all();
        s->cv_work.wait(lk);
      }
      if (s->stop && s->queued == 0) break;
      s->idle = false;
      // ---- the policy
      double best = 0;
      for (int i = 0; i < (int)s->clients.size(); ++i) {
        SchedClient& c = s->clients[i];
        if (c.queue.empty()) continue;
        const double key = s->policy == PW_SCHED_FIFO ? (double)c.queue.front().arrival : c.vtime;
        if (client < 0 || key < best) { client = i; best = key; }
      }
      SchedClient& c = s->clients[client];
      prog = std::move(c.queue.front());
      c.queue.pop_front();
      s->queued--;
      c.vtime += prog.est_us / c.weight;
    }
    while ((int)s->inflight.size() >= s->window) sched_retire(s);
    // ---- enqueue on the executor stream, bracketed by timing events
    SchedInFlight fl;
    fl.client = client;
    fl.n_computations = prog.n_computations;
    SchedResult res;
    const auto t_stall = std::chrono::steady_clock::now();
    bool stalled = false;
    for (;;) {
      {
        std::unique_lock<std::recursive_mutex> api(s->ctx->api_mu);
        const uint64_t saved_owner = s->ctx->current_owner;
        s->ctx->current_owner = s->clients[client].owner;   // what the program produces belongs to its client
        if (!fl.start) fl.start = sched_event(s);
        if (!fl.stop) fl.stop = sched_event(s);
        if (fl.start) (void)hipEventRecord(fl.start, s->ctx->exec);
        res.status = pw_chain(s->ctx, prog.fns.data(), (int)prog.fns.size(), &prog.in, 1, &res.out, 1, PW_STREAM);
        if (fl.stop) (void)hipEventRecord(fl.stop, s->ctx->exec);
        s->ctx->current_owner = saved_owner;
      }
      if (res.status != PW_ERR_OOM) break;
      // Back-pressure (Section 4.6): other programs' buffers occupy the memory budget.  Stall this one: finish
      // what is in flight, then wait for clients to collect results; give up when nothing can change any more.
      stalled = true;
      if (!s->inflight.empty()) { sched_retire(s); continue; }
      bool hopeless;
      {
        std::lock_guard<std::mutex> lk(s->mu);
        hopeless = (s->results.empty() && s->collecting == 0) || s->stop || s->clients[client].failed;   // nothing left to wait for
      }
      if (hopeless || std::chrono::steady_clock::now() - t_stall > std::chrono::seconds(20)) break;
      std::this_thread::sleep_for(std::chrono::microseconds(50));
    }
    if (stalled) {
      std::lock_guard<std::mutex> lk(s->mu);
      s->stalls++;
      s->stalled_ms += std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t_stall).count();
    }
    s->inflight.push_back(fl);
    {
      std::lock_guard<std::mutex> lk(s->mu);
      s->results[prog.ticket] = res;
      SchedClient& c = s->clients[client];
      c.programs++;
      if (res.status == PW_OK) c.computations += prog.n_computations;
    }
    s->cv_done.notify_all();
  }
  while (!s->inflight.empty()) sched_retire(s);
  std::lock_guard<std::mutex> lk(s->mu);
  s->idle = true;
  s->cv_done.notify_all();
}

void sched_shutdown(pw_sched* s) {
  {
    std::lock_guard<std::mutex> lk(s->mu);
    s->stop = true;
  }
  s->cv_work.notify_all();
  if (s->thread.joinable()) s->thread.join();
  // results nobody collected: give their futures back
  for (auto& kv : s->results)
    if (kv.second.status == PW_OK && kv.second.out) (void)pw_future_release(s->ctx, kv.second.out);
  s->results.clear();
  for (hipEvent_t e : s->timing_events) (void)hipEventDestroy(e);
  if (s->epoch) (void)hipEventDestroy(s->epoch);
}

}  // namespace

pw_status pw_sched_create(pw_ctx* c, int policy, int max_in_flight, pw_sched** out) {
  if (!c || !out) return PW_ERR_INVALID;
  PW_API_LOCK(c);
  if (policy != PW_SCHED_FIFO && policy != PW_SCHED_PROPORTIONAL) return fail(c, PW_ERR_INVALID, "unknown scheduling policy");
  if (max_in_flight < 1 || max_in_flight > 1024) return fail(c, PW_ERR_INVALID, "programs in flight must be within [1, 1024]");
  pw_sched* s = new pw_sched();
  s->ctx = c;
  s->policy = policy;
  s->window = max_in_flight;
  if (hipEventCreate(&s->epoch) != hipSuccess || hipEventRecord(s->epoch, c->exec) != hipSuccess) {
    if (s->epoch) (void)hipEventDestroy(s->epoch);
    delete s;
    return fail(c, PW_ERR_DEVICE, "could not create the scheduler's timing events");
  }
  static std::atomic<uint64_t> next_id{1};
  s->id = next_id.fetch_add(1) & 0x7FFFFFFFu;
  s->thread = std::thread(sched_loop, s);
  c->scheds.push_back(s);
  *out = s;
  return PW_OK;
}

pw_status pw_sched_destroy(pw_sched* s) {
  if (!s) return PW_ERR_INVALID;
  pw_ctx* c = s->ctx;
  sched_shutdown(s);
  {
    PW_API_LOCK(c);
    for (size_t i = 0; i < c->scheds.size(); ++i)
      if (c->scheds[i] == s) { c->scheds.erase(c->scheds.begin() + i); break; }
  }
  delete s;
  return PW_OK;
}

pw_status pw_sched_add_client(pw_sched* s, double weight, int* client) {
  if (!s || !client || !(weight > 0.0) || weight > 1e6) return PW_ERR_INVALID;
  std::lock_guard<std::mutex> lk(s->mu);
  if (s->clients.size() >= 1024) return PW_ERR_INVALID;
  SchedClient c;
  c.weight = weight;
  // a newcomer starts level with the least-served client, not with a credit for the past
  bool any = false;
  for (auto& o : s->clients)
    if (!any || o.vtime < c.vtime) { c.vtime = o.vtime; any = true; }
  c.owner = (1ull << 63) | (s->id << 32) | (uint64_t)s->clients.size();
  s->clients.push_back(c);
  *client = (int)s->clients.size() - 1;
  return PW_OK;
}

pw_status pw_sched_client_fail(pw_sched* s, int client, int64_t* objects_released) {
  if (!s) return PW_ERR_INVALID;
  uint64_t owner;
  {
    std::lock_guard<std::mutex> lk(s->mu);
    if (client < 0 || client >= (int)s->clients.size()) return PW_ERR_INVALID;
    SchedClient& c = s->clients[client];
    c.failed = true;
    owner = c.owner;
    // programs that never reached the device are dropped; whoever waits for them learns why
    for (auto& p : c.queue) {
      SchedResult r;
      r.status = PW_ERR_POISONED;
      s->results[p.ticket] = r;
      s->queued--;
    }
    c.queue.clear();
    // results of this client that nobody collected are collected with its other objects below
    for (auto& kv : s->results)
      if (kv.second.status == PW_OK && kv.second.out) {
        FutureRec* f = nullptr;
        {
          std::unique_lock<std::recursive_mutex> api(s->ctx->api_mu);
          f = future_get(s->ctx, kv.second.out);
          if (f && f->owner == owner) { kv.second.status = PW_ERR_POISONED; kv.second.out = 0; }
        }
      }
  }
  s->cv_done.notify_all();
  return pw_owner_collect(s->ctx, owner, objects_released);
}

pw_status pw_sched_stalls(pw_sched* s, int64_t* programs_stalled, double* stalled_ms) {
  if (!s) return PW_ERR_INVALID;
  std::lock_guard<std::mutex> lk(s->mu);
  if (programs_stalled) *programs_stalled = s->stalls;
  if (stalled_ms) *stalled_ms = s->stalled_ms;
  return PW_OK;
}

pw_status pw_sched_submit(pw_sched* s, int client, const pw_fn* fns, int n_fns, pw_future in, uint64_t* ticket) {
  if (!s || !fns || !ticket || n_fns < 1 || n_fns > 4096) return PW_ERR_INVALID;
  SchedProgram p;
  p.fns.assign(fns, fns + n_fns);
  p.in = in;
  {
    // cost estimate from the compiled functions (busy time where known, a launch's worth otherwise)
    PW_API_LOCK(s->ctx);
    for (int i = 0; i < n_fns; ++i) {
      FnRec* f = fn_get(s->ctx, fns[i]);
      if (!f) return fail(s->ctx, PW_ERR_INVALID, "function %d of the program is not a live handle", i);
      p.est_us += 3.0 + (double)f->busy_us * f->reps;
      p.n_computations += f->reps;
    }
    if (!future_get(s->ctx, in)) return fail(s->ctx, PW_ERR_INVALID, "input is not a live future");
  }
  std::lock_guard<std::mutex> lk(s->mu);
  if (client < 0 || client >= (int)s->clients.size()) return PW_ERR_INVALID;
  if (s->stop) return PW_ERR_INVALID;
  SchedClient& c = s->clients[client];
  if (c.failed) return PW_ERR_INVALID;
  if (c.queue.empty() && s->policy == PW_SCHED_PROPORTIONAL) {
    // back from idle: no credit for time not used
    bool any = false;
    double floor_v = 0;
    for (auto& o : s->clients)
      if (!o.queue.empty() && (!any || o.vtime < floor_v)) { floor_v = o.vtime; any = true; }
    if (any && c.vtime < floor_v) c.vtime = floor_v;
  }
  p.ticket = s->next_ticket++;
  p.arrival = s->next_arrival++;
  *ticket = p.ticket;
  s->outstanding[p.ticket] = false;
  c.queue.push_back(std::move(p));
  s->queued++;
  s->cv_work.notify_one();
  return PW_OK;
}

pw_status pw_sched_wait(pw_sched* s, uint64_t ticket, void* host_dst, size_t bytes) {
  if (!s) return PW_ERR_INVALID;
  SchedResult r;
  {
    std::unique_lock<std::mutex> lk(s->mu);
    auto o = s->outstanding.find(ticket);
    if (o == s->outstanding.end() || o->second) return PW_ERR_INVALID;   // unknown, collected already, or being waited for
    o->second = true;
    s->cv_done.wait(lk, [&] { return s->results.count(ticket) != 0 || s->stop; });
    s->outstanding.erase(ticket);
    auto it = s->results.find(ticket);
    if (it == s->results.end()) return PW_ERR_INVALID;   // the scheduler was shut down first
    r = it->second;
    s->results.erase(it);
    if (r.status == PW_OK) s->collecting++;
  }
  if (r.status != PW_OK) return r.status;
  pw_status st = pw_await(s->ctx, r.out, host_dst, bytes);
  (void)pw_future_release(s->ctx, r.out);
  {
    std::lock_guard<std::mutex> lk(s->mu);
    s->collecting--;
  }
  return st;
}

pw_status pw_sched_drain(pw_sched* s) {
  if (!s) return PW_ERR_INVALID;
  std::unique_lock<std::mutex> lk(s->mu);
  s->cv_done.wait(lk, [&] { return (s->queued == 0 && s->idle) || s->stop; });
  return PW_OK;
}

pw_status pw_sched_client_stats(pw_sched* s, int client, int64_t* programs, int64_t* computations, double* device_ms) {
  if (!s) return PW_ERR_INVALID;
  std::lock_guard<std::mutex> lk(s->mu);
  if (client < 0 || client >= (int)s->clients.size()) return PW_ERR_INVALID;
  if (programs) *programs = s->clients[client].programs;
  if (computations) *computations = s->clients[client].computations;
  if (device_ms) *device_ms = s->clients[client].device_ms;
  return PW_OK;
}

pw_status pw_sched_trace(pw_sched* s, pw_sched_slice* out, int capacity, int* n) {
  if (!s || !n || capacity < 0 || (capacity > 0 && !out)) return PW_ERR_INVALID;
  std::lock_guard<std::mutex> lk(s->mu);
  const int k = std::min<int>(capacity, (int)s->trace.size());
  for (int i = 0; i < k; ++i) out[i] = s->trace[i];
  *n = (int)s->trace.size();
  return PW_OK;
}

pw_status pw_train_step(pw_ctx* c, pw_fn step_fn, pw_future tokens, pw_future* loss_out) {
  PW_API_LOCK(c);
  if (!c || !loss_out) return PW_ERR_INVALID;
  FnRec* fn = fn_get(c, step_fn);
  if (!fn || fn->desc.kind != PW_FN_LM_TRAIN_STEP) return fail(c, PW_ERR_INVALID, "not a train-step function");
  return pw_run_fn(c, step_fn, &tokens, 1, loss_out, 1);
}

// ---- futures -----------------------------------------------------------------------------------------

pw_status pw_await(pw_ctx* c, pw_future h, void* host_dst, size_t bytes) {
  if (!c) return PW_ERR_INVALID;
  PW_API_LOCK(c);
  FutureRec* f = future_get(c, h);
  if (!f) return fail(c, PW_ERR_INVALID, "bad future handle");
  if (bytes > f->bytes) return fail(c, PW_ERR_SHAPE, "asked for %zu bytes of a %zu-byte future", bytes, f->bytes);
  // Block without holding the lock (other threads keep dispatching); the extra reference keeps the record and
  // its event alive meanwhile.
  f->refcount++;
  hipEvent_t ev = f->event;
  hipStream_t exec = c->exec;
  api_lk_.unlock();
  hipError_t e = ev ? hipEventSynchronize(ev) : hipStreamSynchronize(exec);
  api_lk_.lock();
  f = future_get(c, h);   // the table may have been reallocated
  if (!f) return fail(c, PW_ERR_POISONED, "the future was garbage-collected with its owner while being waited for");
  pw_status st = PW_OK;
  if (e != hipSuccess) st = fail(c, PW_ERR_DEVICE, "waiting for the future: %s", hipGetErrorString(e));
  if (st == PW_OK && f->host_poison) st = fail(c, PW_ERR_POISONED, "future depends on a failed producer");
  if (st == PW_OK)
    for (auto& p : f->poison)
      if (__atomic_load_n(&p->words[1], __ATOMIC_ACQUIRE)) { st = fail(c, PW_ERR_POISONED, "a pending input was poisoned or timed out"); break; }
  if (st == PW_OK && host_dst && bytes) {
    if (hipMemcpyAsync(host_dst, f->buf, bytes, hipMemcpyDeviceToHost, c->io) != hipSuccess || hipStreamSynchronize(c->io) != hipSuccess)
      st = fail(c, PW_ERR_DEVICE, "copy to the host failed");
  }
  future_drop(c, h);
  return st;
}

pw_status pw_future_from_host(pw_ctx* c, const void* src, const pw_tensor_spec* spec, pw_future* out) {
  PW_API_LOCK(c);
  if (!c || !src || !spec || !out) return PW_ERR_INVALID;
  if (!spec_ok(*spec)) return fail(c, PW_ERR_INVALID, "malformed spec");
  void* buf;
  size_t cls;
  pw_status st = pool_alloc(c, spec_bytes(*spec), &buf, &cls);
  if (st != PW_OK) return st;
  if (spec_bytes(*spec)) {
    hipError_t e = hipMemcpyAsync(buf, src, spec_bytes(*spec), hipMemcpyHostToDevice, c->exec);
    if (e != hipSuccess) { pool_free(c, buf, cls); return fail(c, PW_ERR_DEVICE, "H2D copy: %s", hipGetErrorString(e)); }
  }
  FutureRec* f;
  future_new(c, &f, out);
  f->buf = buf; f->pool_bytes = cls; f->bytes = spec_bytes(*spec); f->spec = *spec; f->owns = true;
  return PW_OK;
}

pw_status pw_future_wrap_device(pw_ctx* c, void* dev_ptr, const pw_tensor_spec* spec, pw_future* out) {
  PW_API_LOCK(c);
  if (!c || !dev_ptr || !spec || !out) return PW_ERR_INVALID;
  if (!spec_ok(*spec)) return fail(c, PW_ERR_INVALID, "malformed spec");
  FutureRec* f;
  future_new(c, &f, out);
  f->buf = dev_ptr; f->bytes = spec_bytes(*spec); f->spec = *spec; f->owns = false;
  return PW_OK;
}

pw_status pw_future_pending(pw_ctx* c, const pw_tensor_spec* spec, pw_future* out) {
  PW_API_LOCK(c);
  if (!c || !spec || !out) return PW_ERR_INVALID;
  if (!spec_ok(*spec)) return fail(c, PW_ERR_INVALID, "malformed spec");
  const size_t bytes = spec_bytes(*spec);
  if (bytes > (1ull << 30)) return fail(c, PW_ERR_UNSUPPORTED, "pending futures are limited to 1 GiB");
  void* buf;
  size_t cls;
  pw_status st = pool_alloc(c, bytes, &buf, &cls);
  if (st != PW_OK) return st;
  std::shared_ptr<GateWords> gw = words_get(c);
  void* staging = nullptr;
  auto& sp = c->staging_pool[size_class(bytes)];
  if (!sp.empty()) { staging = sp.back(); sp.pop_back(); }
  else if (hipHostMalloc(&staging, size_class(bytes), hipHostMallocDefault) != hipSuccess) staging = nullptr;
  hipEvent_t ev = nullptr, order = nullptr;
  if (!gw || !staging || event_get(c, &ev) != PW_OK || event_get(c, &order) != PW_OK) {
    pool_free(c, buf, cls);
    if (staging) sp.push_back(staging);
    if (ev) c->event_pool.push_back(ev);
    return fail(c, PW_ERR_OOM, "could not set up a gate");
  }
  // The buffer may have been used by work already enqueued on the executor stream: the gate stream's
  // copy into it must come after that work.
  hipError_t e = hipEventRecord(order, c->exec);
  if (e == hipSuccess) e = hipStreamWaitEvent(c->gate, order, 0);
  c->event_pool.push_back(order);
  if (e == hipSuccess) e = launch_gate(c->gate, gw->words, gw->words + 1, (uint64_t)c->gate_timeout_ms * 100000ull);
  if (e == hipSuccess && bytes) e = launch_copy_bytes(c->gate, staging, buf, (int64_t)bytes);
  if (e == hipSuccess) e = hipEventRecord(ev, c->gate);
  if (e != hipSuccess) {
    __atomic_store_n(&gw->words[0], 2u, __ATOMIC_RELEASE);
    pool_free(c, buf, cls);
    sp.push_back(staging);
    c->event_pool.push_back(ev);
    return fail(c, PW_ERR_DEVICE, "gate launch: %s", hipGetErrorString(e));
  }
  FutureRec* f;
  future_new(c, &f, out);
  f->buf = buf; f->pool_bytes = cls; f->bytes = bytes; f->spec = *spec; f->owns = true;
  f->on_gate_stream = true; f->pending = true; f->event = ev; f->gate = gw; f->staging = staging;
  f->poison.push_back(gw);
  return PW_OK;
}

pw_status pw_future_resolve(pw_ctx* c, pw_future h, const void* host_src) {
  PW_API_LOCK(c);
  if (!c) return PW_ERR_INVALID;
  FutureRec* f = future_get(c, h);
  if (!f) return fail(c, PW_ERR_INVALID, "bad future handle");
  if (!f->pending) return fail(c, PW_ERR_INVALID, "future is not pending");
  f->pending = false;
  if (!host_src) {
    f->host_poison = true;
    __atomic_store_n(&f->gate->words[0], 2u, __ATOMIC_RELEASE);
    return PW_OK;
  }
  std::memcpy(f->staging, host_src, f->bytes);
  __atomic_store_n(&f->gate->words[0], 1u, __ATOMIC_RELEASE);
  return PW_OK;
}

pw_status pw_future_query(pw_ctx* c, pw_future h) {
  PW_API_LOCK(c);
  if (!c) return PW_ERR_INVALID;
  FutureRec* f = future_get(c, h);
  if (!f) return fail(c, PW_ERR_INVALID, "bad future handle");
  if (f->host_poison) return PW_ERR_POISONED;
  hipError_t e = f->event ? hipEventQuery(f->event) : hipStreamQuery(c->exec);
  if (e == hipErrorNotReady) return PW_ERR_NOT_READY;
  if (e != hipSuccess) return fail(c, PW_ERR_DEVICE, "query: %s", hipGetErrorString(e));
  for (auto& p : f->poison)
    if (__atomic_load_n(&p->words[1], __ATOMIC_ACQUIRE)) return PW_ERR_POISONED;
  return PW_OK;
}

pw_status pw_future_spec(pw_ctx* c, pw_future h, pw_tensor_spec* out) {
  PW_API_LOCK(c);
  if (!c || !out) return PW_ERR_INVALID;
  FutureRec* f = future_get(c, h);
  if (!f) return fail(c, PW_ERR_INVALID, "bad future handle");
  *out = f->spec;
  return PW_OK;
}

pw_status pw_future_device_ptr(pw_ctx* c, pw_future h, void** out) {
  PW_API_LOCK(c);
  if (!c || !out) return PW_ERR_INVALID;
  FutureRec* f = future_get(c, h);
  if (!f) return fail(c, PW_ERR_INVALID, "bad future handle");
  *out = f->buf;
  return PW_OK;
}

pw_status pw_future_retain(pw_ctx* c, pw_future h) {
  PW_API_LOCK(c);
  if (!c) return PW_ERR_INVALID;
  FutureRec* f = future_get(c, h);
  if (!f) return fail(c, PW_ERR_INVALID, "bad future handle");
  f->refcount++;
  return PW_OK;
}

pw_status pw_future_release(pw_ctx* c, pw_future h) {
  PW_API_LOCK(c);
  if (!c) return PW_ERR_INVALID;
  FutureRec* f = future_get(c, h);
  if (!f) return fail(c, PW_ERR_INVALID, "bad future handle");
  if (f->refcount == 1 && f->on_gate_stream && f->event) {
    // its buffer is written by the gate stream: make sure that write is over before the buffer is reused
    if (f->pending) __atomic_store_n(&f->gate->words[0], 2u, __ATOMIC_RELEASE);
    (void)hipStreamWaitEvent(c->exec, f->event, 0);
  }
  future_drop(c, h);
  return PW_OK;
}

// ---- model -------------------------------------------------------------------------------------------

pw_status pw_model_create(pw_ctx* c, const pw_lm_config* cfg, pw_model** out) {
  if (!c || !cfg || !out) return PW_ERR_INVALID;
  std::string why;
  if (!model_config_ok(*cfg, &why)) return fail(c, PW_ERR_UNSUPPORTED, "%s", why.c_str());
  Model* m = nullptr;
  hipError_t e = model_create(*cfg, c->exec, &m, &why);
  if (e != hipSuccess) return fail(c, e == hipErrorOutOfMemory ? PW_ERR_OOM : PW_ERR_DEVICE, "%s", why.c_str());
  c->models.push_back(m);
  *out = new pw_model{c, m};
  return PW_OK;
}

pw_status pw_model_destroy(pw_model* pm) {
  if (!pm) return PW_ERR_INVALID;
  pw_ctx* c = pm->ctx;
  (void)hipStreamSynchronize(c->exec);
  for (size_t i = 0; i < c->models.size(); ++i)
    if (c->models[i] == pm->impl) {
      c->models.erase(c->models.begin() + i);
      model_destroy(pm->impl);
      break;
    }
  for (auto& f : c->fns)
    if (f.live && f.model == pm->impl) f.live = false;   // functions of a dead model die with it
  delete pm;
  return PW_OK;
}

// Parameter-table access shared by the two kinds of model (both keep their state in a ModelBase).
static float* part_base(ModelBase* m, int part) {
  switch (part) {
    case PW_PARAMS: return m->w;
    case PW_GRADS: return m->g;
    case PW_ADAM_M: return m->m;
    case PW_ADAM_V: return m->v;
  }
  return nullptr;
}
static pw_status state_param_info(ModelBase* m, int64_t idx, char* name, int cap, int64_t* numel) {
  if (idx < 0 || idx >= (int64_t)m->params.size()) return PW_ERR_INVALID;
  const ParamInfo& p = m->params[idx];
  if (name && cap > 0) snprintf(name, cap, "%s", p.name.c_str());
  if (numel) *numel = p.numel;
  return PW_OK;
}
static pw_status state_import(pw_ctx* c, ModelBase* m, int part, int64_t idx, const float* src, int src_on_device) {
  if (!src || idx < 0 || idx >= (int64_t)m->params.size()) return PW_ERR_INVALID;
  float* base = part_base(m, part);
  if (!base) return fail(c, PW_ERR_INVALID, "this model has no such part");
  const ParamInfo& p = m->params[idx];
  PW_HIP(c, hipMemcpyAsync(base + p.offset, src, (size_t)p.numel * 4, src_on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, c->exec));
  if (part == PW_PARAMS) {
    hipError_t e = model_state_refresh_lowp(m, p.offset, p.numel);
    if (e != hipSuccess) return fail(c, PW_ERR_DEVICE, "bf16 refresh: %s", hipGetErrorString(e));
  }
  PW_HIP(c, hipStreamSynchronize(c->exec));
  return PW_OK;
}
static pw_status state_export(pw_ctx* c, ModelBase* m, int part, int64_t idx, float* dst) {
  if (!dst || idx < 0 || idx >= (int64_t)m->params.size()) return PW_ERR_INVALID;
  float* base = part_base(m, part);
  if (!base) return fail(c, PW_ERR_INVALID, "this model has no such part");
  const ParamInfo& p = m->params[idx];
  PW_HIP(c, hipStreamSynchronize(c->exec));
  PW_HIP(c, hipMemcpy(dst, base + p.offset, (size_t)p.numel * 4, hipMemcpyDeviceToHost));
  return PW_OK;
}
// Copies n elements of a device array in the activation type out as fp32, after draining the executor stream.
static pw_status export_activation(pw_ctx* c, const void* src, int64_t n, bool is_bf16, float* dst) {
  PW_HIP(c, hipStreamSynchronize(c->exec));
  if (!is_bf16) {
    PW_HIP(c, hipMemcpy(dst, src, (size_t)n * 4, hipMemcpyDeviceToHost));
    return PW_OK;
  }
  float* tmp = nullptr;
  PW_HIP(c, hipMalloc(&tmp, (size_t)n * 4));
  hipError_t e = launch_bf16_to_f32(c->exec, src, tmp, n);
  if (e == hipSuccess) e = hipStreamSynchronize(c->exec);
  if (e == hipSuccess) e = hipMemcpy(dst, tmp, (size_t)n * 4, hipMemcpyDeviceToHost);
  (void)hipFree(tmp);
  if (e != hipSuccess) return fail(c, PW_ERR_DEVICE, "activation export: %s", hipGetErrorString(e));
  return PW_OK;
}

int64_t pw_model_param_count(pw_model* pm) { return pm ? (int64_t)pm->impl->params.size() : -1; }
pw_status pw_model_param_info(pw_model* pm, int64_t idx, char* name, int cap, int64_t* numel) {
  return pm ? state_param_info(pm->impl, idx, name, cap, numel) : PW_ERR_INVALID;
}
pw_status pw_model_import(pw_model* pm, int part, int64_t idx, const float* src, int src_on_device) {
  return pm ? state_import(pm->ctx, pm->impl, part, idx, src, src_on_device) : PW_ERR_INVALID;
}
pw_status pw_model_export(pw_model* pm, int part, int64_t idx, float* dst) {
  return pm ? state_export(pm->ctx, pm->impl, part, idx, dst) : PW_ERR_INVALID;
}

pw_status pw_model_zero_grads(pw_model* pm) {
  if (!pm) return PW_ERR_INVALID;
  if (model_zero_grads(pm->impl) != hipSuccess) return fail(pm->ctx, PW_ERR_DEVICE, "%s", pm->impl->error.c_str());
  return PW_OK;
}

pw_status pw_model_apply_optimizer(pw_model* pm) {
  if (!pm) return PW_ERR_INVALID;
  if (model_apply_optimizer(pm->impl) != hipSuccess) return fail(pm->ctx, PW_ERR_DEVICE, "%s", pm->impl->error.c_str());
  return PW_OK;
}

pw_status pw_model_export_activation(pw_model* pm, const char* name, int mb, float* dst, int64_t numel) {
  if (!pm || !name || !dst) return PW_ERR_INVALID;
  pw_ctx* c = pm->ctx;
  Model* m = pm->impl;
  if (mb < 0 || mb >= m->cfg.n_microbatch) return fail(c, PW_ERR_INVALID, "micro-batch index out of range");
  const int64_t N = m->N(), d = m->cfg.d_model;
  const void* src = nullptr;
  int64_t n = 0;
  int dt = PW_F32;
  const std::string s(name);
  if (s == "x_out") { src = m->slots[mb].x_out; n = N * d; }
  else if (s == "dlogits" && m->logits) { src = m->logits; n = N * m->cfg.vocab; dt = m->act_dtype(); }
  else if (s == "dx_in") { src = m->dx_a; n = N * d; }
  else return fail(c, PW_ERR_INVALID, "unknown activation name");
  if (numel != n) return fail(c, PW_ERR_SHAPE, "activation has %lld elements", (long long)n);
  return export_activation(c, src, n, dt != PW_F32, dst);
}

double pw_model_step_flops(const pw_lm_config* cfg) { return cfg ? model_step_flops(*cfg) : 0.0; }

// ---- encoder-decoder model -------------------------------------------------------------------------------

pw_status pw_encdec_create(pw_ctx* c, const pw_encdec_config* cfg, pw_encdec** out) {
  if (!c || !cfg || !out) return PW_ERR_INVALID;
  std::string why;
  if (!encdec_config_ok(*cfg, &why)) return fail(c, PW_ERR_UNSUPPORTED, "%s", why.c_str());
  EncDec* m = nullptr;
  hipError_t e = encdec_create(*cfg, c->exec, &m, &why);
  if (e != hipSuccess) return fail(c, e == hipErrorOutOfMemory ? PW_ERR_OOM : PW_ERR_DEVICE, "%s", why.c_str());
  c->encdecs.push_back(m);
  *out = new pw_encdec{c, m};
  return PW_OK;
}

pw_status pw_encdec_destroy(pw_encdec* pm) {
  if (!pm) return PW_ERR_INVALID;
  pw_ctx* c = pm->ctx;
  (void)hipStreamSynchronize(c->exec);
  for (size_t i = 0; i < c->encdecs.size(); ++i)
    if (c->encdecs[i] == pm->impl) {
      c->encdecs.erase(c->encdecs.begin() + i);
      encdec_destroy(pm->impl);
      break;
    }
  for (auto& f : c->fns)
    if (f.live && f.encdec == pm->impl) f.live = false;   // functions of a dead model die with it
  delete pm;
  return PW_OK;
}

int64_t pw_encdec_param_count(pw_encdec* pm) { return pm ? (int64_t)pm->impl->params.size() : -1; }
pw_status pw_encdec_param_info(pw_encdec* pm, int64_t idx, char* name, int cap, int64_t* numel) {
  return pm ? state_param_info(pm->impl, idx, name, cap, numel) : PW_ERR_INVALID;
}
pw_status pw_encdec_import(pw_encdec* pm, int part, int64_t idx, const float* src, int src_on_device) {
  return pm ? state_import(pm->ctx, pm->impl, part, idx, src, src_on_device) : PW_ERR_INVALID;
}
pw_status pw_encdec_export(pw_encdec* pm, int part, int64_t idx, float* dst) {
  return pm ? state_export(pm->ctx, pm->impl, part, idx, dst) : PW_ERR_INVALID;
}

pw_status pw_encdec_export_activation(pw_encdec* pm, const char* name, float* dst, int64_t numel) {
  if (!pm || !name || !dst) return PW_ERR_INVALID;
  pw_ctx* c = pm->ctx;
  EncDec* m = pm->impl;
  if (std::string(name) != "dlogits") return fail(c, PW_ERR_INVALID, "unknown activation name");
  const int64_t n = (int64_t)m->Nt() * m->cfg.vocab;
  if (numel != n) return fail(c, PW_ERR_SHAPE, "activation has %lld elements", (long long)n);
  return export_activation(c, m->logits, n, m->bf16 != 0, dst);
}

double pw_encdec_step_flops(const pw_encdec_config* cfg) { return cfg ? encdec_step_flops(*cfg) : 0.0; }

// ---- single kernels ------------------------------------------------------------------------------------

#define PW_OP(c, expr)                                                                               \
  do {                                                                                               \
    if (!(c)) return PW_ERR_INVALID;                                                                 \
    hipError_t e_ = (expr);                                                                          \
    if (e_ == hipErrorInvalidValue) return fail(c, PW_ERR_INVALID, "arguments rejected by the launcher"); \
    if (e_ == hipErrorNotSupported) return fail(c, PW_ERR_UNSUPPORTED, "not supported");            \
    if (e_ != hipSuccess) return fail(c, PW_ERR_DEVICE, "%s", hipGetErrorString(e_));               \
    return PW_OK;                                                                                    \
  } while (0)

static GemmArgs gemm_args_of(const pw_gemm_args* a) {
  GemmArgs g{};
  g.dtype = a->dtype; g.a_kmajor = a->a_kmajor; g.b_kmajor = a->b_kmajor;
  g.M = a->M; g.N = a->N; g.K = a->K; g.lda = a->lda; g.ldb = a->ldb; g.ldc = a->ldc;
  g.epilogue = a->epilogue; g.out_dtype = a->out_dtype; g.accumulate = a->accumulate;
  g.A = a->A; g.B = a->B; g.bias = a->bias; g.aux = a->aux; g.C = a->C; g.C2 = a->C2;
  g.b_colsum = a->b_colsum;
  return g;
}
pw_status pw_op_gemm(pw_ctx* c, const pw_gemm_args* a) {
  if (!c || !a) return PW_ERR_INVALID;
  PW_OP(c, launch_gemm(c->exec, gemm_args_of(a)));
}
pw_status pw_op_gemm_pair(pw_ctx* c, const pw_gemm_args* a0, const pw_gemm_args* a1) {
  if (!c || !a0 || !a1) return PW_ERR_INVALID;
  PW_OP(c, launch_gemm_pair(c->exec, gemm_args_of(a0), gemm_args_of(a1)));
}
pw_status pw_op_gemm_group(pw_ctx* c, const pw_gemm_args* a, int n) {
  if (!c || !a || n < 1 || n > 3) return PW_ERR_INVALID;
  GemmArgs g[3];
  for (int i = 0; i < n; ++i) g[i] = gemm_args_of(&a[i]);
  PW_OP(c, launch_gemm_group(c->exec, g, n));
}
pw_status pw_op_embedding_fwd(pw_ctx* c, const int32_t* tokens, const float* wte, const float* wpe, float* x, int B, int T, int d, int V) {
  PW_OP(c, launch_embedding_fwd(c->exec, tokens, wte, wpe, x, B, T, d, V));
}
pw_status pw_op_embedding_bwd(pw_ctx* c, const int32_t* tokens, const float* dx, float* dwte, float* dwpe, int B, int T, int d, int V) {
  PW_OP(c, launch_embedding_bwd(c->exec, tokens, dx, dwte, dwpe, B, T, d, V));
}
pw_status pw_op_layernorm_fwd(pw_ctx* c, int dtype, const float* x, const float* g, const float* b, void* y, float* mean, float* rstd, int N, int d) {
  PW_OP(c, launch_layernorm_fwd(c->exec, dtype, x, g, b, y, mean, rstd, N, d));
}
pw_status pw_op_layernorm_bwd(pw_ctx* c, int dtype, const void* dy, const float* x, const float* g, const float* mean, const float* rstd,
                              const float* dres, float* dx, void* dx_lp, float* dg, float* db, float* dxsum, float* ws, int N, int d, int accumulate) {
  PW_OP(c, launch_layernorm_bwd(c->exec, dtype, dy, x, g, mean, rstd, dres, dx, dx_lp, dg, db, dxsum, ws, N, d, accumulate));
}
int64_t pw_layernorm_bwd_ws_floats(int N, int d) { return layernorm_bwd_ws_floats(N, d); }
pw_status pw_op_attention_fwd(pw_ctx* c, int dtype, const void* qkv, void* o, float* lse, int B, int T, int H, int hd) {
  PW_OP(c, launch_attention_fwd(c->exec, dtype, qkv, o, lse, B, T, H, hd));
}
pw_status pw_op_attention_bwd(pw_ctx* c, int dtype, const void* qkv, const void* o, const void* dout, const float* lse, float* delta,
                              void* dqkv, int B, int T, int H, int hd) {
  PW_OP(c, launch_attention_bwd(c->exec, dtype, qkv, o, dout, lse, delta, dqkv, B, T, H, hd));
}
static MhaArgs mha_args_of(const pw_mha_args* a) {
  return MhaArgs{a->dtype, a->q, a->k, a->v, a->ldq, a->ldkv, a->B, a->Tq, a->Tk, a->H, a->hd, a->causal};
}
pw_status pw_op_mha_fwd(pw_ctx* c, const pw_mha_args* a, void* o, void* o_lo, float* lse) {
  if (!a) return PW_ERR_INVALID;
  PW_OP(c, launch_mha_fwd(c->exec, mha_args_of(a), o, o_lo, lse));
}
pw_status pw_op_mha_bwd(pw_ctx* c, const pw_mha_args* a, const void* o, const void* o_lo, const void* dout, const float* lse,
                        float* delta, void* dq, int64_t lddq, void* dk, void* dv, int64_t lddkv) {
  if (!a) return PW_ERR_INVALID;
  PW_OP(c, launch_mha_bwd(c->exec, mha_args_of(a), o, o_lo, dout, lse, delta, dq, lddq, dk, dv, lddkv));
}
pw_status pw_op_softmax_xent(pw_ctx* c, int dtype, void* z, const int32_t* tokens, float* loss, float* row_loss, int B, int T, int V) {
  PW_OP(c, launch_softmax_xent(c->exec, dtype, z, tokens, loss, row_loss, B, T, V));
}
pw_status pw_op_colsum(pw_ctx* c, int dtype, const void* in, float* out, float* ws, int64_t rows, int64_t cols, int accumulate) {
  PW_OP(c, launch_colsum(c->exec, dtype, in, out, ws, rows, cols, accumulate));
}
int64_t pw_colsum_ws_floats(int64_t rows, int64_t cols) { return colsum_ws_floats(rows, cols); }
pw_status pw_op_sgd(pw_ctx* c, float* w, const float* g, int64_t n, float lr) { PW_OP(c, launch_sgd(c->exec, w, g, n, lr)); }
pw_status pw_op_adam(pw_ctx* c, float* w, float* m, float* v, const float* g, void* w_bf16, int64_t n, float lr, float beta1, float beta2,
                     float eps, int t) {
  PW_OP(c, launch_adam(c->exec, w, m, v, g, w_bf16, n, lr, beta1, beta2, eps, t, nullptr));
}

pw_status pw_profile_begin(pw_ctx* c) {
  if (!c) return PW_ERR_INVALID;
  gemm_profile_begin();
  return PW_OK;
}
pw_status pw_profile_pause(pw_ctx* c) {
  if (!c) return PW_ERR_INVALID;
  gemm_profile_pause();
  return PW_OK;
}
pw_status pw_profile_end(pw_ctx* c, int64_t* launches, double* total_ms, double* total_flops) {
  if (!c) return PW_ERR_INVALID;
  hipError_t e = gemm_profile_end(launches, total_ms, total_flops);
  if (e != hipSuccess) return fail(c, PW_ERR_DEVICE, "profile read: %s", hipGetErrorString(e));
  return PW_OK;
}

}  // extern "C"
