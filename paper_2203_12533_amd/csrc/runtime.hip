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
#include "runtime_internal.hpp"

namespace {


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

// A completion word and a token no earlier user of the word can have written (tokens are unique per context; a late
// write of an old token to a recycled word is overwritten, in stream order, by the new owner's).
std::shared_ptr<GateWords> done_word_get(pw_ctx* c, uint32_t* token) {
  if (c->free_done_words.empty()) {
    uint32_t* slab = nullptr;
    if (hipHostMalloc((void**)&slab, 4096, hipHostMallocDefault) != hipSuccess) return nullptr;
    c->word_slabs.push_back(slab);   // freed with the gate slabs at context destruction
    for (int i = 0; i < 4096 / 64; ++i) c->free_done_words.push_back(slab + i * 16);
  }
  uint32_t* w = c->free_done_words.back();
  c->free_done_words.pop_back();
  if (++c->done_seq == 0) ++c->done_seq;
  *token = c->done_seq;
  pw_ctx* ctx = c;
  return std::shared_ptr<GateWords>(new GateWords{w}, [ctx](GateWords* g) {
    ctx->free_done_words.push_back(g->words);
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
  f->done.reset();
  f->live = false;
  c->live_futures--;
  c->free_futures.push_back((uint32_t)(h & 0xFFFFFFFFu) - 1);
}


bool is_scalar_kind(int k) { return k >= PW_FN_ADD_CONST && k <= PW_FN_BUSY_CHAIN; }   // one fp32 input, one output

// Launch the body of one function on the executor stream.  in/out are device pointers.
// Whether a launch of fn can carry a completion word (see FutureRec::done).
bool fn_signals_completion(const FnRec* fn) { return is_scalar_kind(fn->desc.kind) && scalar_fn_one_block(spec_numel(fn->desc.in[0])); }

pw_status fn_launch(pw_ctx* c, FnRec* fn, void* const* in, void* const* out, uint32_t* done = nullptr, uint32_t token = 0) {
  const int k = fn->desc.kind;
  if (is_scalar_kind(k)) {
    hipError_t e = launch_scalar_fn(c->exec, k, (const float*)in[0], (float*)out[0], spec_numel(fn->desc.in[0]), fn->cst, fn->busy_us, fn->reps,
                                    done, token);
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
// Host-side part of a stage function that runs inside a HIP graph (fresh capture or cached replay alike).
pw_status graph_host_effects(pw_ctx* c, const FnRec* fn) {
  const int k = fn->desc.kind;
  if ((k == PW_FN_STAGE_FWD || k == PW_FN_STAGE_BWD) && fn->model &&
      model_before_graph(fn->model, k == PW_FN_STAGE_BWD) != hipSuccess)
    return fail(c, PW_ERR_DEVICE, "%s", fn->model->error.c_str());
  return PW_OK;
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
  if (gemm_init() != hipSuccess || attention_dma_init() != hipSuccess || layernorm_bwd_static_init(device) != hipSuccess) {
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
  std::shared_ptr<GateWords> done;
  uint32_t done_token = 0;
  if (st == PW_OK && fn_signals_completion(fn)) done = done_word_get(c, &done_token);   // none to be had: the event alone
  if (st == PW_OK) st = fn_launch(c, fn, ibuf, obuf, done ? done->words : nullptr, done_token);
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
      f->done = done;
      f->done_token = done_token;
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
  // A HIP-graph launch has a fixed cost worth about eight stream launches of a trivial kernel: shorter chains of
  // single-kernel functions are enqueued as stream launches (same launches, same results).
  if (mode == PW_GRAPH && n_fns < 8) {
    bool single_kernels = true;
    for (int i = 0; i < n_fns; ++i) single_kernels = single_kernels && (is_scalar_kind(recs[i]->desc.kind) || recs[i]->desc.kind == PW_FN_ADD2);
    if (single_kernels) mode = PW_STREAM;
  }
  if (mode == PW_SEQUENTIAL) {
    // This baseline waits on the host for every link.  An input that hangs on an unresolved pending future would
    // make it wait - holding the context's lock, so that pw_future_resolve could not get in - until the gate gives up.
    for (int i = 0; i < n_in; ++i)
      for (auto& gw : fin[i]->poison)
        if (__atomic_load_n(&gw->words[0], __ATOMIC_ACQUIRE) == 0u)
          return fail(c, PW_ERR_NOT_READY, "PW_SEQUENTIAL waits for every link: input %d depends on a pending future that has not been resolved", i);
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

  // Stream launches whose last link is a one-block elementwise function: that launch also signals completion to the host.
  std::shared_ptr<GateWords> done;
  uint32_t done_token = 0;
  if (mode != PW_GRAPH && n_out == 1 && fn_signals_completion(recs[n_fns - 1])) done = done_word_get(c, &done_token);
  auto enqueue_all = [&](bool sync_each) -> pw_status {
    void* ibuf[8];
    void* obuf[8];
    for (int j = 0; j < n_in; ++j) ibuf[j] = fin[j]->buf;
    for (int i = 0; i < n_fns; ++i) {
      for (size_t j = 0; j < plan_bufs[i].size(); ++j) obuf[j] = plan_bufs[i][j].p;
      const bool last = i + 1 == n_fns && done;
      pw_status s2 = fn_launch(c, recs[i], ibuf, obuf, last ? done->words : nullptr, last ? done_token : 0);
      if (s2 != PW_OK) return s2;
      if (sync_each && hipStreamSynchronize(c->exec) != hipSuccess) return fail(c, PW_ERR_DEVICE, "stream synchronize failed");
      for (size_t j = 0; j < plan_bufs[i].size(); ++j) ibuf[j] = obuf[j];
    }
    return PW_OK;
  };

  if (mode == PW_GRAPH) {
    for (int i = 0; i < n_fns; ++i)
      if ((st = graph_host_effects(c, recs[i])) != PW_OK) { release_all(); return st; }
    std::string key;
    key.append((const char*)fns, sizeof(pw_fn) * n_fns);
    for (int j = 0; j < n_in; ++j) key.append((const char*)&fin[j]->buf, sizeof(void*));
    for (auto& v : plan_bufs)
      for (auto& b : v) key.append((const char*)&b.p, sizeof(void*));
    auto it = c->graphs.find(key);
    if (it == c->graphs.end()) {
      if (c->graphs.size() >= 256) {   // bounded cache: drop everything rather than grow without limit
        (void)hipStreamSynchronize(c->exec);   // a replay enqueued by an earlier call may not have run yet
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
      f->done = done;
      f->done_token = done_token;
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
  for (size_t i = 0; i < p->nodes.size(); ++i) {   // the nodes hold snapshots of their functions: a model may be gone since
    const FnRec& fn = p->nodes[i].fn;
    if ((fn.model && !model_alive(c, fn.model)) || (fn.encdec && !encdec_alive(c, fn.encdec)))
      return fail(c, PW_ERR_INVALID, "node %zu runs a function of a model that has been destroyed", i);
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
    for (int i = 0; i < n_nodes; ++i)
      if ((st = graph_host_effects(c, &p->nodes[i].fn)) != PW_OK) { release_outputs(); return st; }
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
  // Readiness alone (nothing to copy out) of a future with a completion word: poll the word for a while - it arrives
  // microseconds before the stream's event does - and fall back to the event if it does not show up.
  const std::shared_ptr<GateWords> done = (host_dst && bytes) ? nullptr : f->done;
  const uint32_t done_token = f->done_token;
  api_lk_.unlock();
  bool signalled = false;
  if (done) {
    const auto t0 = std::chrono::steady_clock::now();
    for (int spin = 0; !signalled; ++spin) {
      signalled = __atomic_load_n(&done->words[0], __ATOMIC_ACQUIRE) == done_token;
      if (!signalled && (spin & 255) == 255 && std::chrono::steady_clock::now() - t0 > std::chrono::microseconds(200)) break;
    }
  }
  hipError_t e = signalled ? hipSuccess : ev ? hipEventSynchronize(ev) : hipStreamSynchronize(exec);
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
  const bool signalled = f->done && __atomic_load_n(&f->done->words[0], __ATOMIC_ACQUIRE) == f->done_token;
  hipError_t e = signalled ? hipSuccess : f->event ? hipEventQuery(f->event) : hipStreamQuery(c->exec);
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

}  // extern "C"
