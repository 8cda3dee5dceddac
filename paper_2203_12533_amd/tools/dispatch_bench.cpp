// Dispatch micro-benchmarks of Section 5.1 on one GPU, driven through the C boundary only (no Python, no HIP
// calls of its own).  Prints one JSON object per line.
//
//  * "overhead_masking": the trivial computation of the first micro-benchmark is given a tunable duration and
//    enqueued four ways - op by op (a client call and an await per computation), chained (one client call for 128
//    nodes; as stream launches and as one HIP-graph replay), and fused (128 computations inside one node).  Fused
//    has no per-computation dispatch cost at all, so it plays the part of the multi-controller system in the
//    paper's comparison; the smallest duration at which Chained reaches 95 % / 99 % of Fused throughput is the
//    analogue of the "smallest computation that masks the single-controller overhead".
//  * "parallel_vs_sequential": one trivial computation per pipeline stage, every stage on an executor of its own,
//    handed out all at once or one after the other (the second micro-benchmark of the section).
//  * "multi_tenancy": several client threads submit programs (chains of 16 computations) to the central scheduler
//    (Section 5.2): aggregate throughput against the number of clients and the computation size, and the split
//    of device time between four clients under proportional-share weights 1:1:1:1 and 1:2:4:8.
//
// Build: g++ -O2 -std=c++17 -I include dispatch_bench.cpp -L <dir of libpw.so> -lpw -Wl,-rpath,<dir> -o dispatch_bench
#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <atomic>
#include <string>
#include <thread>
#include <vector>

#include "pw.h"

namespace {

double now_s() { return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count(); }

#define CHECK(expr)                                                                              \
  do {                                                                                           \
    pw_status st_ = (expr);                                                                      \
    if (st_ != PW_OK) {                                                                          \
      std::fprintf(stderr, "%s failed (%d): %s\n", #expr, (int)st_, ctx ? pw_last_error(ctx) : ""); \
      std::exit(1);                                                                              \
    }                                                                                            \
  } while (0)

pw_ctx* ctx = nullptr;
constexpr int kN = 128;

pw_fn compile(int kind, float c, float busy_us, int reps) {
  pw_fn_desc d{};
  d.kind = kind;
  d.n_in = d.n_out = 1;
  d.in[0].dtype = d.out[0].dtype = PW_F32;
  d.in[0].rank = d.out[0].rank = 1;
  d.in[0].dims[0] = d.out[0].dims[0] = kN;
  float params[3] = {c, busy_us, (float)reps};
  d.params = params;
  d.params_bytes = (kind == PW_FN_BUSY ? 2 : kind == PW_FN_BUSY_CHAIN ? 3 : 1) * sizeof(float);
  pw_fn f;
  CHECK(pw_compile_fn(ctx, &d, &f));
  return f;
}

pw_future input() {
  std::vector<float> x(kN);
  for (int i = 0; i < kN; ++i) x[i] = 0.001f * i;
  pw_tensor_spec s{};
  s.dtype = PW_F32;
  s.rank = 1;
  s.dims[0] = kN;
  pw_future f;
  CHECK(pw_future_from_host(ctx, x.data(), &s, &f));
  CHECK(pw_await(ctx, f, nullptr, 0));
  return f;
}

// Runs `program` (which enqueues `count` computations and waits for the last) until ~budget seconds have passed;
// returns the best computations per second over the repetitions (after two warm-up runs).
template <class F>
double throughput(int count, double budget_s, F program) {
  program();
  program();
  double best = 0;
  const double t_end = now_s() + budget_s;
  int reps = 0;
  do {
    const double t0 = now_s();
    program();
    const double dt = now_s() - t0;
    best = std::max(best, count / dt);
    ++reps;
  } while ((now_s() < t_end && reps < 200) || reps < 3);
  return best;
}

}  // namespace

int main(int argc, char** argv) {
  bool quick = false, gaps = false;
  for (int i = 1; i < argc; ++i) {
    quick = quick || std::strcmp(argv[i], "--quick") == 0;
    gaps = gaps || std::strcmp(argv[i], "--gaps") == 0;
  }
  if (pw_ctx_create(0, nullptr, &ctx) != PW_OK) {
    std::fprintf(stderr, "no usable gfx950 GPU\n");
    return 2;
  }
  if (gaps) {
    // For a kernel trace (rocprofv3 --kernel-trace -- dispatch_bench --gaps): the same chain of 128 trivial
    // computations dispatched four ways, 20 times each (then two pipelines, below), the phases 100 ms apart so that the trace can be cut at the
    // pauses.  The device-side launch gap of a mode is next.start - previous.end between consecutive kernels of a chain.
    constexpr int L = 128, reps = 20;
    pw_future x = input();
    pw_fn one = compile(PW_FN_ADD_CONST, 1.f, 0.f, 1);
    std::vector<pw_fn> chain(L, one);
    const char* names[4] = {"chained_stream", "chained_graph", "sequential", "op_by_op"};
    for (int phase = 0; phase < 4; ++phase) {
      std::this_thread::sleep_for(std::chrono::milliseconds(100));
      const double t0 = now_s();
      for (int r = 0; r < reps + 2; ++r) {      // two warm-up chains (graph capture) count as part of the phase
        if (phase < 3) {
          pw_future out;
          CHECK(pw_chain(ctx, chain.data(), L, &x, 1, &out, 1, phase == 0 ? PW_STREAM : phase == 1 ? PW_GRAPH : PW_SEQUENTIAL));
          CHECK(pw_await(ctx, out, nullptr, 0));
          CHECK(pw_future_release(ctx, out));
        } else {
          pw_future cur = x;
          for (int i = 0; i < L; ++i) {
            pw_future out;
            CHECK(pw_run_fn(ctx, one, &cur, 1, &out, 1));
            CHECK(pw_await(ctx, out, nullptr, 0));
            if (i) CHECK(pw_future_release(ctx, cur));
            cur = out;
          }
          CHECK(pw_future_release(ctx, cur));
        }
      }
      std::printf("{\"bench\": \"launch_gaps\", \"phase\": %d, \"mode\": \"%s\", \"chains\": %d, \"chain_length\": %d, "
                  "\"wall_us_per_computation\": %.3f}\n", phase, names[phase], reps + 2, L, (now_s() - t0) * 1e6 / ((reps + 2) * L));
    }
    // Two more phases for the cost of a dependency that crosses executors: a pipeline of 64 stages, every stage on an
    // executor (stream + host thread) of its own, parallel dispatch - and the same pipeline with all stages on
    // executor 0, where the dependency is stream order.
    CHECK(pw_ctx_set_executors(ctx, 64));
    {
      constexpr int stages = 64;
      std::vector<pw_fn> fns(stages, one);
      const char* pnames[2] = {"pipeline_64_executors", "pipeline_1_executor"};
      for (int phase = 0; phase < 2; ++phase) {
        std::vector<int32_t> where(stages);
        for (int i = 0; i < stages; ++i) where[i] = phase == 0 ? i : 0;
        std::this_thread::sleep_for(std::chrono::milliseconds(100));
        const double t0 = now_s();
        for (int r = 0; r < reps + 2; ++r) {
          pw_future out;
          CHECK(pw_pipeline(ctx, fns.data(), where.data(), stages, x, &out, PW_DISPATCH_PARALLEL));
          CHECK(pw_await(ctx, out, nullptr, 0));
          CHECK(pw_future_release(ctx, out));
        }
        std::printf("{\"bench\": \"launch_gaps\", \"phase\": %d, \"mode\": \"%s\", \"chains\": %d, \"chain_length\": %d, "
                    "\"wall_us_per_computation\": %.3f}\n", 4 + phase, pnames[phase], reps + 2, stages, (now_s() - t0) * 1e6 / ((reps + 2) * stages));
      }
    }
    CHECK(pw_future_release(ctx, x));
    pw_ctx_destroy(ctx);
    return 0;
  }
  CHECK(pw_ctx_set_executors(ctx, 64));
  const double budget = quick ? 0.05 : 0.25;
  constexpr int L = 128;
  pw_future x = input();
  float got[kN];

  // ---- overhead masking -----------------------------------------------------------------------------
  const std::vector<float> durations = quick ? std::vector<float>{0, 2, 5, 10, 20, 50, 100, 500}
                                             : std::vector<float>{0, 1, 2, 3, 5, 7, 10, 15, 20, 30, 50, 75, 100, 200, 500, 1000, 2000};
  double mask95 = -1, mask99 = -1, mask95_graph = -1, mask99_graph = -1;
  for (float us : durations) {
    pw_fn one = compile(PW_FN_BUSY, 1.f, us, 1), fused = compile(PW_FN_BUSY_CHAIN, 1.f, us, L);
    std::vector<pw_fn> chain(L, one);
    auto run_chain = [&](int mode) {
      pw_future out;
      CHECK(pw_chain(ctx, chain.data(), L, &x, 1, &out, 1, mode));
      CHECK(pw_await(ctx, out, nullptr, 0));
      CHECK(pw_future_release(ctx, out));
    };
    const double t_fused = throughput(L, budget, [&] {
      pw_future out;
      CHECK(pw_run_fn(ctx, fused, &x, 1, &out, 1));
      CHECK(pw_await(ctx, out, nullptr, 0));
      CHECK(pw_future_release(ctx, out));
    });
    const double t_stream = throughput(L, budget, [&] { run_chain(PW_STREAM); });
    const double t_graph = throughput(L, budget, [&] { run_chain(PW_GRAPH); });
    const double t_seq = throughput(L, budget, [&] { run_chain(PW_SEQUENTIAL); });
    const double t_op = throughput(L, budget, [&] {
      pw_future cur = x;
      for (int i = 0; i < L; ++i) {
        pw_future out;
        CHECK(pw_run_fn(ctx, one, &cur, 1, &out, 1));
        CHECK(pw_await(ctx, out, nullptr, 0));
        if (i) CHECK(pw_future_release(ctx, cur));
        cur = out;
      }
      CHECK(pw_future_release(ctx, cur));
    });
    std::printf("{\"bench\": \"overhead_masking\", \"computation_us\": %g, \"chain_length\": %d, \"computations_per_s\": "
                "{\"fused\": %.0f, \"chained_stream\": %.0f, \"chained_graph\": %.0f, \"sequential\": %.0f, \"op_by_op\": %.0f}, "
                "\"chained_over_fused\": {\"stream\": %.4f, \"graph\": %.4f}}\n",
                us, L, t_fused, t_stream, t_graph, t_seq, t_op, t_stream / t_fused, t_graph / t_fused);
    std::fflush(stdout);
    if (mask95 < 0 && t_stream >= 0.95 * t_fused) mask95 = us;
    if (mask99 < 0 && t_stream >= 0.99 * t_fused) mask99 = us;
    if (t_stream < 0.95 * t_fused) mask95 = -1;     // must hold for every longer computation too
    if (t_stream < 0.99 * t_fused) mask99 = -1;
    if (mask95_graph < 0 && t_graph >= 0.95 * t_fused) mask95_graph = us;
    if (mask99_graph < 0 && t_graph >= 0.99 * t_fused) mask99_graph = us;
    if (t_graph < 0.95 * t_fused) mask95_graph = -1;
    if (t_graph < 0.99 * t_fused) mask99_graph = -1;
    CHECK(pw_fn_release(ctx, one));
    CHECK(pw_fn_release(ctx, fused));
  }
  std::printf("{\"bench\": \"overhead_masking_summary\", \"smallest_computation_us_for_chained_to_reach\": "
              "{\"stream_95pct\": %g, \"stream_99pct\": %g, \"graph_95pct\": %g, \"graph_99pct\": %g}, "
              "\"note\": \"-1: not reached within the sweep\"}\n", mask95, mask99, mask95_graph, mask99_graph);

  // ---- parallel vs sequential dispatch over pipeline stages ----------------------------------------
  // prep_us: emulated host-side preparation per node (0: only what this runtime really spends).
  struct Case { float computation_us; int prep_us; };
  const std::vector<Case> cases = quick ? std::vector<Case>{{0.f, 0}, {20.f, 50}} : std::vector<Case>{{0.f, 0}, {20.f, 0}, {0.f, 50}, {100.f, 50}};
  for (const Case& cs : cases) {
    CHECK(pw_ctx_set_executor_prep_us(ctx, cs.prep_us));
    pw_fn one = compile(PW_FN_BUSY, 1.f, cs.computation_us, 1);
    for (int stages : {1, 2, 4, 8, 16, 32, 64}) {
      std::vector<pw_fn> fns(stages, one);
      std::vector<int32_t> where(stages);
      for (int i = 0; i < stages; ++i) where[i] = i;
      double tp[2], host_us[2] = {1e30, 1e30};
      for (int mode = 0; mode < 2; ++mode)
        tp[mode] = throughput(stages, budget, [&] {
          pw_future out;
          const double t0 = now_s();
          CHECK(pw_pipeline(ctx, fns.data(), where.data(), stages, x, &out, mode == 0 ? PW_DISPATCH_PARALLEL : PW_DISPATCH_SEQUENTIAL));
          host_us[mode] = std::min(host_us[mode], (now_s() - t0) * 1e6 / stages);
          CHECK(pw_await(ctx, out, got, sizeof got));
          CHECK(pw_future_release(ctx, out));
        });
      if (got[0] != (float)stages) {   // x[0] = 0, one addition of 1 per stage
        std::fprintf(stderr, "wrong pipeline result %g for %d stages\n", got[0], stages);
        return 1;
      }
      std::printf("{\"bench\": \"parallel_vs_sequential\", \"computation_us\": %g, \"host_prep_us\": %d, \"stages\": %d, "
                  "\"computations_per_s\": {\"parallel\": %.0f, \"sequential\": %.0f}, \"parallel_over_sequential\": %.3f, "
                  "\"enqueue_call_us_per_stage\": {\"parallel\": %.2f, \"sequential\": %.2f}}\n",
                  cs.computation_us, cs.prep_us, stages, tp[0], tp[1], tp[0] / tp[1], host_us[0], host_us[1]);
      std::fflush(stdout);
    }
    CHECK(pw_fn_release(ctx, one));
  }
  CHECK(pw_ctx_set_executor_prep_us(ctx, 0));
  // ---- multi-tenancy ----------------------------------------------------------------------------------
  {
    constexpr int kProg = 16;   // computations per program
    const double run_s = quick ? 0.1 : 0.3;
    auto run_clients = [&](pw_sched* sched, const std::vector<int>& ids, pw_fn fn, int outstanding, std::vector<long>& done) {
      std::vector<pw_fn> prog(kProg, fn);
      std::atomic<bool> stop{false};
      std::vector<std::thread> th;
      done.assign(ids.size(), 0);
      for (size_t k = 0; k < ids.size(); ++k)
        th.emplace_back([&, k] {
          std::vector<uint64_t> tickets;
          while (!stop.load(std::memory_order_relaxed)) {
            while ((int)tickets.size() < outstanding) {
              uint64_t t;
              if (pw_sched_submit(sched, ids[k], prog.data(), kProg, x, &t) != PW_OK) return;
              tickets.push_back(t);
            }
            if (pw_sched_wait(sched, tickets.front(), nullptr, 0) != PW_OK) return;
            tickets.erase(tickets.begin());
            done[k] += kProg;
          }
          for (uint64_t t : tickets) (void)pw_sched_wait(sched, t, nullptr, 0);
        });
      std::this_thread::sleep_for(std::chrono::duration<double>(run_s));
      stop.store(true);
      for (auto& t : th) t.join();
    };
    for (float us : quick ? std::vector<float>{0.f, 330.f} : std::vector<float>{0.f, 10.f, 100.f, 330.f}) {
      pw_fn fn = compile(PW_FN_BUSY, 1.f, us, 1);
      // one client alone, straight on the context (no scheduler): the yardstick
      std::vector<pw_fn> prog(kProg, fn);
      const double alone = throughput(kProg, budget, [&] {
        pw_future out;
        CHECK(pw_chain(ctx, prog.data(), kProg, &x, 1, &out, 1, PW_STREAM));
        CHECK(pw_await(ctx, out, nullptr, 0));
        CHECK(pw_future_release(ctx, out));
      });
      for (int n_clients : {1, 2, 4, 8, 16}) {
        pw_sched* sched;
        CHECK(pw_sched_create(ctx, PW_SCHED_FIFO, 8, &sched));
        std::vector<int> ids(n_clients);
        for (int& id : ids) CHECK(pw_sched_add_client(sched, 1.0, &id));
        std::vector<long> done;
        const double t0 = now_s();
        run_clients(sched, ids, fn, 1, done);
        const double dt = now_s() - t0;
        long total = 0;
        for (long d : done) total += d;
        CHECK(pw_sched_destroy(sched));
        std::printf("{\"bench\": \"multi_tenancy\", \"computation_us\": %g, \"clients\": %d, \"programs_of\": %d, "
                    "\"aggregate_computations_per_s\": %.0f, \"one_client_without_scheduler\": %.0f, \"device_limit\": %.0f}\n",
                    us, n_clients, kProg, total / dt, alone, us > 0 ? 1e6 / us : 0.0);
        std::fflush(stdout);
      }
      CHECK(pw_fn_release(ctx, fn));
    }
    pw_fn fn = compile(PW_FN_BUSY, 1.f, 330.f / kProg, 1);   // programs of 0.33 ms
    for (int set = 0; set < 2; ++set) {
      const double w[2][4] = {{1, 1, 1, 1}, {1, 2, 4, 8}};
      pw_sched* sched;
      CHECK(pw_sched_create(ctx, PW_SCHED_PROPORTIONAL, 2, &sched));
      std::vector<int> ids(4);
      for (int k = 0; k < 4; ++k) CHECK(pw_sched_add_client(sched, w[set][k], &ids[k]));
      std::vector<long> done;
      run_clients(sched, ids, fn, 4, done);
      CHECK(pw_sched_drain(sched));
      double ms[4], total = 0;
      for (int k = 0; k < 4; ++k) {
        int64_t p, c;
        CHECK(pw_sched_client_stats(sched, ids[k], &p, &c, &ms[k]));
        total += ms[k];
      }
      CHECK(pw_sched_destroy(sched));
      std::printf("{\"bench\": \"proportional_share\", \"program_ms\": 0.33, \"weights\": [%g, %g, %g, %g], "
                  "\"device_time_share\": [%.3f, %.3f, %.3f, %.3f], \"device_busy_fraction\": %.3f}\n",
                  w[set][0], w[set][1], w[set][2], w[set][3], ms[0] / total, ms[1] / total, ms[2] / total, ms[3] / total,
                  total / 1e3 / run_s);
      std::fflush(stdout);
    }
    CHECK(pw_fn_release(ctx, fn));
  }
  CHECK(pw_future_release(ctx, x));
  CHECK(pw_ctx_destroy(ctx));
  return 0;
}
