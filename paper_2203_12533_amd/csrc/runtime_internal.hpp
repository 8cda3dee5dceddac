// Internal records of the future/dispatch runtime, shared by its translation units (runtime.hip,
// runtime_sched.hip, runtime_models.hip).  Nothing here is part of the C boundary: include/pw.h only names
// pw_ctx, pw_model, pw_encdec, pw_program and pw_sched as opaque types.
#pragma once

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

namespace pw {
namespace rt {


inline size_t dtype_size(int dt) { return dt == PW_BF16 ? 2 : 4; }

inline bool spec_ok(const pw_tensor_spec& s) {
  if (s.dtype < PW_F32 || s.dtype > PW_I32 || s.rank < 0 || s.rank > 4) return false;
  for (int i = 0; i < s.rank; ++i)
    if (s.dims[i] < 0 || s.dims[i] > (1LL << 40)) return false;
  return true;
}
inline int64_t spec_numel(const pw_tensor_spec& s) {
  int64_t n = 1;
  for (int i = 0; i < s.rank; ++i) n *= s.dims[i];
  return n;
}
inline size_t spec_bytes(const pw_tensor_spec& s) { return (size_t)spec_numel(s) * dtype_size(s.dtype); }
// 0 same, PW_ERR_DTYPE or PW_ERR_SHAPE otherwise
inline pw_status spec_match(const pw_tensor_spec& a, const pw_tensor_spec& b) {
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
  // Completion word (futures produced by a one-block elementwise launch on the executor stream): the kernel writes
  // done_token to done->words[0] when its output is complete, so pw_await can poll pinned memory instead of waiting
  // for the stream's end-of-kernel event to reach the host.
  std::shared_ptr<GateWords> done;
  uint32_t done_token = 0;
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

}  // namespace rt
}  // namespace pw

// (internal header of three translation units: the directives keep the record names short in all of them)
using namespace pw;
using namespace pw::rt;

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
  // completion words: a pool of their own - a kernel may write its word after the future was released, which a
  // word recycled as a gate flag would read as "resolved"
  std::vector<uint32_t*> free_done_words;
  uint32_t done_seq = 0;
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
namespace pw {
namespace rt {
struct ProgNode {
  FnRec fn;            // snapshot: the handle may be released after tracing
  pw_fn handle = 0;    // only part of the graph-cache key
  int n_in = 0, in[8] = {0};
  int first_out = 0;
};
}  // namespace rt
}  // namespace pw
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
namespace pw {
namespace rt {
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
}  // namespace rt
}  // namespace pw

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

namespace pw {
namespace rt {

// Records the message on the context (read back by pw_last_error) and returns the status.
inline pw_status fail(pw_ctx* c, pw_status st, const char* fmt, ...) {
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

// Handles are (generation << 32) | (slot + 1): a stale handle finds a different generation and gives null.
inline FutureRec* future_get(pw_ctx* c, pw_future h) {
  const uint32_t idx = (uint32_t)(h & 0xFFFFFFFFu), gen = (uint32_t)(h >> 32);
  if (idx == 0 || idx > c->futures.size()) return nullptr;
  FutureRec& f = c->futures[idx - 1];
  return (f.live && f.gen == gen) ? &f : nullptr;
}
inline FnRec* fn_get(pw_ctx* c, pw_fn h) {
  const uint32_t idx = (uint32_t)(h & 0xFFFFFFFFu), gen = (uint32_t)(h >> 32);
  if (idx == 0 || idx > c->fns.size()) return nullptr;
  FnRec& f = c->fns[idx - 1];
  return (f.live && f.gen == gen) ? &f : nullptr;
}

}  // namespace rt
}  // namespace pw
