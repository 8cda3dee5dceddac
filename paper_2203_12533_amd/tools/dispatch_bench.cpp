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
//
// Build: g++ -O2 -std=c++17 -I include dispatch_bench.cpp -L <dir of libpw.so> -lpw -Wl,-rpath,<dir> -o dispatch_bench
#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
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
  bool quick = false;
  for (int i = 1; i < argc; ++i) quick = quick || std::strcmp(argv[i], "--quick") == 0;
  if (pw_ctx_create(0, nullptr, &ctx) != PW_OK) {
    std::fprintf(stderr, "no usable gfx950 GPU\n");
    return 2;
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
  CHECK(pw_future_release(ctx, x));
  CHECK(pw_ctx_destroy(ctx));
  return 0;
}
