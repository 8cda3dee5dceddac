// Multi-tenant scheduler of the dispatch runtime (Section 4.4: one scheduler per island that orders the
// programs of all clients; Section 5.2: FIFO and proportional-share policies).  The records are described in
// runtime_internal.hpp; the calls are declared in include/pw.h.
#include "runtime_internal.hpp"

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
    uint64_t client_owner = 0;
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
      client_owner = c.owner;   // copied under the lock: pw_sched_add_client may move the vector
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
        s->ctx->current_owner = client_owner;   // what the program produces belongs to its client
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

extern "C" {

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

}  // extern "C"
