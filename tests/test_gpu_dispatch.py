"""Dispatch layer on the GPU: chained compiled functions consuming futures (Sections 3, 4.4, 4.5, 5.1)."""
import os
import time

import numpy as np
import pytest

from paper_2203_12533_amd import binding as pwb
from paper_2203_12533_amd import inputs as I

pytestmark = pytest.mark.gpu
GOLD = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def ctx():
    c = pwb.Context(0)
    yield c
    c.close()


@pytest.mark.parametrize("mode", [pwb.PW_STREAM, pwb.PW_GRAPH, pwb.PW_SEQUENTIAL])
@pytest.mark.parametrize("L", [1, 8, 32, 128])
def test_chain_on_pending_input_is_exact(ctx, orc, L, mode):
    x = I.dispatch_input()
    add1 = ctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, 128, 1.0)
    want = orc.chain_add(x, L)
    for rep in range(3):                       # replays of a cached graph must stay right
        xin = x + np.float32(rep)
        want = orc.chain_add(xin, L)
        if mode == pwb.PW_SEQUENTIAL:
            # this baseline waits for every link to finish, so its input has to exist already
            f_in = ctx.future_from_host(xin)
            (f_out,) = ctx.chain([add1] * L, [f_in], 1, mode)
        else:
            f_in = ctx.future_pending(pwb.PW_F32, (128,))
            (f_out,) = ctx.chain([add1] * L, [f_in], 1, mode)
            # the whole chain is enqueued although its input does not exist yet
            assert ctx.future_query(f_out) == pwb.PW_ERR_NOT_READY
            ctx.future_resolve(f_in, xin)
        got = ctx.await_(f_out)
        assert np.array_equal(got, want), (L, mode, rep)
        assert ctx.future_query(f_out) == pwb.PW_OK
        ctx.future_release(f_in)
        ctx.future_release(f_out)
    ctx.fn_release(add1)


@pytest.mark.parametrize("L", [1, 8])
def test_readiness_through_the_completion_word_is_not_early_and_not_lost(ctx, orc, L):
    """A one-block elementwise launch tells the host it is done through a word in pinned memory, which pw_await polls
    when nothing has to be copied out.  Readiness must not be reported before a pending input was resolved, the value
    behind it must be complete, and words recycled over many futures must keep their futures apart."""
    import threading, time
    x = I.dispatch_input()
    add1 = ctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, 128, 1.0)
    # (a) not early: the input is resolved 50 ms after the wait has begun
    f_in = ctx.future_pending(pwb.PW_F32, (128,))
    (f_out,) = ctx.chain([add1] * L, [f_in], 1, pwb.PW_STREAM)
    t0 = time.perf_counter()
    th = threading.Thread(target=lambda: (time.sleep(0.05), ctx.future_resolve(f_in, x)))
    th.start()
    ctx.await_(f_out, fetch=False)
    waited = time.perf_counter() - t0
    th.join()
    assert waited >= 0.045, waited
    assert np.array_equal(ctx.await_(f_out), orc.chain_add(x, L))
    ctx.future_release(f_in)
    ctx.future_release(f_out)
    # (b) many short-lived futures, op by op and as chains, some released without ever being awaited
    f = ctx.future_from_host(x)
    for i in range(300):
        (g,) = ctx.run_fn(add1, [f]) if i % 2 else ctx.chain([add1], [f], 1, pwb.PW_GRAPH)
        if i % 3:
            ctx.await_(g, fetch=False)
            assert ctx.future_query(g) == pwb.PW_OK
        ctx.future_release(f)
        f = g
    ctx.await_(f, fetch=False)
    assert np.array_equal(ctx.await_(f), orc.chain_add(x, 300))
    ctx.future_release(f)
    # (c) a function of several blocks has no completion word and goes through the event as before
    big = ctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, 4096, 1.0)
    xb = np.arange(4096, dtype=np.float32)
    fb = ctx.future_from_host(xb)
    (gb,) = ctx.run_fn(big, [fb])
    ctx.await_(gb, fetch=False)
    assert np.array_equal(ctx.await_(gb), xb + np.float32(1.0))
    for h in (fb, gb):
        ctx.future_release(h)
    ctx.fn_release(add1)
    ctx.fn_release(big)


def test_sequential_mode_is_not_given_a_pending_input(ctx):
    """PW_SEQUENTIAL synchronises after every link; with a ready input it must give the same bits."""
    x = I.dispatch_input()
    add1 = ctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, 128, 1.0)
    f_in = ctx.future_from_host(x)
    outs = []
    for mode in (pwb.PW_STREAM, pwb.PW_GRAPH, pwb.PW_SEQUENTIAL):
        (f,) = ctx.chain([add1] * 16, [f_in], 1, mode)
        outs.append(ctx.await_(f))
        ctx.future_release(f)
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
    ctx.future_release(f_in)


def test_sequential_mode_refuses_an_unresolved_input(ctx, orc):
    """The baseline blocks on the host after every link; on an input nobody has resolved yet it would block with the
    context locked until the gate times out.  It is refused up front, nothing is enqueued, and works once resolved."""
    x = I.dispatch_input()
    add1 = ctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, 128, 1.0)
    f_in = ctx.future_pending(pwb.PW_F32, (128,))
    (f_mid,) = ctx.chain([add1], [f_in], 1, pwb.PW_STREAM)          # derived from the pending one
    live0, bytes0 = ctx.stats()
    for f in (f_in, f_mid):
        with pytest.raises(pwb.PwError) as e:
            ctx.chain([add1] * 4, [f], 1, pwb.PW_SEQUENTIAL)
        assert e.value.status == pwb.PW_ERR_NOT_READY
    assert ctx.stats() == (live0, bytes0)
    ctx.future_resolve(f_in, x)
    (f_out,) = ctx.chain([add1] * 4, [f_mid], 1, pwb.PW_SEQUENTIAL)
    assert np.array_equal(ctx.await_(f_out), orc.chain_add(x, 5))      # five sequential fp32 additions
    for f in (f_in, f_mid, f_out):
        ctx.future_release(f)
    ctx.fn_release(add1)


def test_op_by_op_equals_chained(ctx, orc):
    x = I.dispatch_input()
    add1 = ctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, 128, 1.0)
    f = ctx.future_from_host(x)
    for _ in range(32):
        (g,) = ctx.run_fn(add1, [f])
        ctx.future_release(f)
        f = g
    assert np.array_equal(ctx.await_(f), orc.chain_add(x, 32))
    ctx.future_release(f)


def test_figure2_program_with_fan_out(ctx):
    rows = {}
    for line in open(os.path.join(GOLD, "fig2_example.txt")):
        if line.strip() and not line.startswith("#"):
            k, *v = line.split()
            rows[k] = np.array(v, dtype=np.float32)
    n = rows["input"].size
    a = ctx.compile_scalar_fn(pwb.PW_FN_MUL_CONST, n, 2.0)
    b = ctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, n, 1.0)
    c = ctx.compile_scalar_fn(pwb.PW_FN_DIV_CONST, n, 2.0)
    v = ctx.future_pending(pwb.PW_F32, (n,))
    (x,) = ctx.run_fn(a, [v])
    (y,) = ctx.run_fn(b, [x])          # x feeds two consumers
    (cx,) = ctx.run_fn(c, [x])
    (z,) = ctx.run_fn(a, [cx])         # `a` is reused
    assert ctx.future_query(y) == pwb.PW_ERR_NOT_READY and ctx.future_query(z) == pwb.PW_ERR_NOT_READY
    ctx.future_resolve(v, rows["input"])
    assert np.array_equal(ctx.await_(y), rows["y"])
    assert np.array_equal(ctx.await_(z), rows["z"])
    for f in (v, x, y, cx, z):
        ctx.future_release(f)


def test_signature_mismatch_is_rejected_before_any_launch(ctx):
    add128 = ctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, 128, 1.0)
    add64 = ctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, 64, 1.0)
    live0, bytes0 = ctx.stats()
    f64 = ctx.future_from_host(np.zeros(64, np.float32))
    fi = ctx.future_from_host(np.zeros(128, np.int32))
    with pytest.raises(pwb.PwError) as e:
        ctx.run_fn(add128, [f64])
    assert e.value.status == pwb.PW_ERR_SHAPE
    with pytest.raises(pwb.PwError) as e:
        ctx.run_fn(add128, [fi])
    assert e.value.status == pwb.PW_ERR_DTYPE
    with pytest.raises(pwb.PwError) as e:          # link 1 of the chain does not fit link 0's output
        ctx.chain([add64, add128], [f64], 1, pwb.PW_STREAM)
    assert e.value.status == pwb.PW_ERR_SHAPE
    with pytest.raises(pwb.PwError) as e:
        ctx.run_fn(add128, [f64, f64])
    assert e.value.status == pwb.PW_ERR_SHAPE
    with pytest.raises(pwb.PwError) as e:
        ctx.run_fn(12345, [f64])
    assert e.value.status == pwb.PW_ERR_INVALID
    with pytest.raises(pwb.PwError) as e:          # impossible signature at compile time
        ctx.compile_fn(pwb.PW_FN_ADD_CONST, [pwb.make_spec(pwb.PW_F32, (4,))], [pwb.make_spec(pwb.PW_F32, (5,))],
                       np.float32(1).tobytes())
    assert e.value.status == pwb.PW_ERR_SHAPE
    ctx.future_release(f64)
    ctx.future_release(fi)
    assert ctx.stats() == (live0, bytes0)          # the failed calls allocated nothing that stayed


def test_poisoned_and_timed_out_inputs_poison_their_dependents(ctx):
    add1 = ctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, 128, 1.0)
    f_in = ctx.future_pending(pwb.PW_F32, (128,))
    (f_out,) = ctx.chain([add1] * 4, [f_in], 1, pwb.PW_STREAM)
    ctx.future_resolve(f_in, None)                 # the producer "failed"
    with pytest.raises(pwb.PwError) as e:
        ctx.await_(f_out)
    assert e.value.status == pwb.PW_ERR_POISONED
    assert ctx.future_query(f_out) == pwb.PW_ERR_POISONED
    ctx.future_release(f_in)
    ctx.future_release(f_out)
    # a gate nobody resolves gives up by itself after the (here tiny) time limit: every kernel still exits
    ctx.set_gate_timeout_ms(50)
    f_in = ctx.future_pending(pwb.PW_F32, (128,))
    (f_out,) = ctx.run_fn(add1, [f_in])
    t0 = time.time()
    with pytest.raises(pwb.PwError) as e:
        ctx.await_(f_out)
    assert e.value.status == pwb.PW_ERR_POISONED and time.time() - t0 < 5.0
    ctx.set_gate_timeout_ms(20000)
    ctx.future_release(f_in)
    ctx.future_release(f_out)


def test_refcounts_and_pool_reuse(ctx):
    live0, bytes0 = ctx.stats()
    add1 = ctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, 128, 1.0)
    f = ctx.future_from_host(np.ones(128, np.float32))
    ctx.future_retain(f)
    ctx.future_release(f)
    (g,) = ctx.run_fn(add1, [f])                   # still alive after one release
    assert ctx.await_(g)[0] == 2.0
    ctx.future_release(f)
    with pytest.raises(pwb.PwError):               # now it is gone
        ctx.run_fn(add1, [f])
    ctx.future_release(g)
    assert ctx.stats() == (live0, bytes0)
    p1 = []
    for _ in range(3):
        h = ctx.future_from_host(np.ones(128, np.float32))
        p1.append(ctx.future_device_ptr(h))
        ctx.future_release(h)
    assert p1[0] == p1[1] == p1[2]                 # the pool hands the same buffer back


def test_busy_function_and_empty_tensor(ctx):
    busy = ctx.compile_scalar_fn(pwb.PW_FN_BUSY, 128, 1.0, busy_us=200.0)
    f = ctx.future_from_host(np.zeros(128, np.float32))
    t0 = time.time()
    (g,) = ctx.chain([busy] * 10, [f], 1, pwb.PW_STREAM)
    out = ctx.await_(g)
    assert np.array_equal(out, np.full(128, 10.0, np.float32)) and time.time() - t0 > 0.0015
    ctx.future_release(f)
    ctx.future_release(g)
    add0 = ctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, 0, 1.0)
    f = ctx.future_from_host(np.zeros(0, np.float32))
    (g,) = ctx.run_fn(add0, [f])
    assert ctx.await_(g).size == 0
    ctx.future_release(f)
    ctx.future_release(g)


# ---- a chain fused into one node, and chains spread over several executors (Section 5.1) ----------------

@pytest.mark.parametrize("L", [1, 7, 128])
def test_fused_chain_equals_the_chain_of_separate_functions(ctx, orc, L):
    """The "Fused" case: L computations inside one node.  Same L sequential fp32 additions, so same bits."""
    x = I.dispatch_input() * np.float32(3.0)
    fused = ctx.compile_scalar_fn(pwb.PW_FN_BUSY_CHAIN, 128, 1.0, busy_us=2.0, reps=L)
    f_in = ctx.future_pending(pwb.PW_F32, (128,))
    (f_out,) = ctx.run_fn(fused, [f_in])
    ctx.future_resolve(f_in, x)
    assert np.array_equal(ctx.await_(f_out), orc.chain_add(x, L))
    for h in (f_in, f_out):
        ctx.future_release(h)
    ctx.fn_release(fused)
    with pytest.raises(pwb.PwError):
        ctx.compile_scalar_fn(pwb.PW_FN_BUSY_CHAIN, 128, 1.0, busy_us=2.0, reps=0)
    with pytest.raises(pwb.PwError):
        ctx.compile_scalar_fn(pwb.PW_FN_BUSY_CHAIN, 128, 1.0, busy_us=1e6, reps=100)     # more than ten seconds


@pytest.fixture(scope="module")
def pctx():
    c = pwb.Context(0)
    c.set_executors(8)
    yield c
    c.close()


@pytest.mark.parametrize("dispatch", [pwb.PW_DISPATCH_PARALLEL, pwb.PW_DISPATCH_SEQUENTIAL])
@pytest.mark.parametrize("placement", ["round_robin", "one_executor", "blocks_of_3", "back_and_forth"])
def test_pipeline_over_executors_is_exact(pctx, orc, placement, dispatch):
    """Every node on its own executor (or not): the result is the chain's, whatever the placement and the way the
    nodes were handed out; nothing is left allocated afterwards."""
    L, S = 37, 8
    where = {"round_robin": [i % S for i in range(L)], "one_executor": [5] * L,
             "blocks_of_3": [(i // 3) % S for i in range(L)], "back_and_forth": [0 if i % 2 else 7 for i in range(L)]}[placement]
    add1 = pctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, 128, 1.0)
    mul = pctx.compile_scalar_fn(pwb.PW_FN_MUL_CONST, 128, 1.0009765625)
    fns = [add1 if i % 5 else mul for i in range(L)]
    live0, bytes0 = pctx.stats()
    for rep in range(3):
        x = I.dispatch_input() + np.float32(rep)
        want = x.copy()
        for i in range(L):
            want = orc.scalar_fn("add" if i % 5 else "mul", want, 1.0 if i % 5 else 1.0009765625)
        f_in = pctx.future_pending(pwb.PW_F32, (128,))
        f_out = pctx.pipeline(fns, where, f_in, dispatch)
        assert pctx.future_query(f_out) == pwb.PW_ERR_NOT_READY       # enqueued before its input exists
        pctx.future_resolve(f_in, x)
        assert np.array_equal(pctx.await_(f_out), want), (placement, dispatch, rep)
        # the result feeds ordinary functions on the context's own executor afterwards
        (g,) = pctx.run_fn(add1, [f_out])
        assert np.array_equal(pctx.await_(g), orc.scalar_fn("add", want, 1.0))
        for h in (f_in, f_out, g):
            pctx.future_release(h)
    assert pctx.stats() == (live0, bytes0)
    pctx.fn_release(add1)
    pctx.fn_release(mul)


def test_pipeline_rejects_bad_programs_before_enqueuing_and_propagates_poison(pctx):
    add1 = pctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, 128, 1.0)
    add_other = pctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, 64, 1.0)
    f_in = pctx.future_from_host(np.zeros(128, np.float32))
    live0, bytes0 = pctx.stats()
    with pytest.raises(pwb.PwError) as e:
        pctx.pipeline([add1, add1], [0, 8], f_in)                  # there is no executor 8
    assert e.value.status == pwb.PW_ERR_INVALID
    with pytest.raises(pwb.PwError) as e:
        pctx.pipeline([add1, add_other, add1], [0, 1, 2], f_in)    # shapes do not chain
    assert e.value.status == pwb.PW_ERR_SHAPE
    with pytest.raises(pwb.PwError):
        pctx.set_executors(4)                                      # once per context
    assert pctx.stats() == (live0, bytes0)
    pctx.future_release(f_in)
    # a failed producer poisons what the pipeline computes from it
    f_bad = pctx.future_pending(pwb.PW_F32, (128,))
    f_out = pctx.pipeline([add1] * 4, [1, 2, 3, 4], f_bad)
    pctx.future_resolve(f_bad, None)
    with pytest.raises(pwb.PwError) as e:
        pctx.await_(f_out)
    assert e.value.status == pwb.PW_ERR_POISONED
    for h in (f_bad, f_out):
        pctx.future_release(h)
    c2 = pwb.Context(0)
    f = c2.future_from_host(np.zeros(128, np.float32))
    a = c2.compile_scalar_fn(pwb.PW_FN_ADD_CONST, 128, 1.0)
    with pytest.raises(pwb.PwError):
        c2.pipeline([a], [0], f)                                   # executors were never set up
    c2.close()


# ---- several clients, one executor (Sections 4.4 and 5.2) ------------------------------------------------

def test_scheduler_runs_programs_of_concurrent_clients_exactly(orc):
    """Four client threads submit chains of different lengths at once; every program's result is exact, every
    ticket can be waited for from its own thread, nothing stays allocated."""
    import threading
    ctx = pwb.Context(0)
    sched = pwb.Scheduler(ctx, pwb.PW_SCHED_FIFO, max_in_flight=3)
    add1 = ctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, 128, 1.0)
    x = I.dispatch_input()
    f_in = ctx.future_from_host(x)
    live0, bytes0 = ctx.stats()
    errors = []

    def client(cid, length, reps):
        try:
            for r in range(reps):
                t = sched.submit(cid, [add1] * length, f_in)
                got = sched.wait(t, 128)
                if not np.array_equal(got, orc.chain_add(x, length)):
                    errors.append((cid, r))
        except Exception as e:                                # noqa: BLE001 - reported below
            errors.append((cid, repr(e)))

    ids = [sched.add_client(1.0) for _ in range(4)]
    threads = [threading.Thread(target=client, args=(ids[i], 3 + 5 * i, 25)) for i in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    sched.drain()
    assert not errors, errors
    for i, cid in enumerate(ids):
        programs, comps, ms = sched.client_stats(cid)
        assert programs == 25 and comps == 25 * (3 + 5 * i) and ms > 0
    assert ctx.stats() == (live0, bytes0)
    # a program that cannot be enqueued reports its error through its ticket; the scheduler keeps going
    add_other = ctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, 64, 1.0)
    bad = sched.submit(ids[0], [add1, add_other], f_in)
    good = sched.submit(ids[1], [add1], f_in)
    with pytest.raises(pwb.PwError) as e:
        sched.wait(bad)
    assert e.value.status == pwb.PW_ERR_SHAPE
    assert np.array_equal(sched.wait(good, 128), orc.chain_add(x, 1))
    with pytest.raises(pwb.PwError):
        sched.wait(good)                                       # a ticket can be waited for once
    sched.close()
    ctx.close()


@pytest.mark.parametrize("weights", [(1, 1, 1, 1), (1, 2, 4, 8)])
def test_proportional_share_of_device_time(weights):
    """All clients keep work queued; device time (HIP events around every program) splits like the weights.
    FIFO with the same submissions splits evenly whatever the weights."""
    for policy in (pwb.PW_SCHED_PROPORTIONAL, pwb.PW_SCHED_FIFO):
        ctx = pwb.Context(0)
        sched = pwb.Scheduler(ctx, policy, max_in_flight=2)
        busy = ctx.compile_scalar_fn(pwb.PW_FN_BUSY, 128, 1.0, busy_us=100.0)
        f_in = ctx.future_from_host(np.zeros(128, np.float32))
        ids = [sched.add_client(float(w)) for w in weights]
        per_client = 120
        # everything is queued up front, round-robin, so every client stays backlogged while the others are served
        tickets = [sched.submit(ids[i % 4], [busy] * 4, f_in) for i in range(4 * per_client)]
        # look at the schedule once the heaviest client has been served completely
        sched.drain()
        trace = sched.trace()
        assert len(trace) == 4 * per_client
        total = sum(weights)
        if policy == pwb.PW_SCHED_PROPORTIONAL:
            # while all four are backlogged (until the best-served one runs out) time splits like the weights
            n_window = int(per_client * total / max(weights) * 0.9)
            window = trace[:n_window]
            share = [sum(e - s for c, _, s, e in window if c == ids[i]) for i in range(4)]
            for i in range(4):
                want = weights[i] / total
                assert abs(share[i] / sum(share) - want) < 0.25 * want + 0.02, (weights, share)
        else:
            window = trace[:200]
            count = [sum(1 for c, _, _, _ in window if c == ids[i]) for i in range(4)]
            assert max(count) - min(count) <= 2, count                  # arrival order was round-robin
        # slices do not overlap: one program at a time owns the device
        for a, b in zip(trace, trace[1:]):
            assert b[2] >= a[3] - 0.02
        for t in tickets:
            sched.wait(t)
        sched.close()
        ctx.close()


# ---- traced dataflow programs (Section 3, Figure 2) -----------------------------------------------------

def _golden_fig2():
    rows = {}
    for line in open(os.path.join(GOLD, "fig2_example.txt")):
        if line.strip() and not line.startswith("#"):
            k, *v = line.split()
            rows[k] = np.array(v, dtype=np.float32)
    return rows


@pytest.mark.parametrize("mode", [pwb.PW_STREAM, pwb.PW_GRAPH])
def test_traced_figure2_program_runs_from_one_call(ctx, mode):
    """f(v): x = a(v); y = b(x); z = a(c(x)); return (y, z) with a = *2, b = +1, c = /2 - traced once, then each
    run is one client call; the values the paper prints for v = [1, 2] come back, also on graph replays."""
    rows = _golden_fig2()
    n = rows["input"].size
    a = ctx.compile_scalar_fn(pwb.PW_FN_MUL_CONST, n, 2.0)
    b = ctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, n, 1.0)
    c = ctx.compile_scalar_fn(pwb.PW_FN_DIV_CONST, n, 2.0)
    spec = pwb.make_spec(pwb.PW_F32, (n,))
    # values: 0 = v, 1 = x, 2 = y, 3 = c(x), 4 = z
    prog = pwb.Program(ctx, [spec], [(a, [0]), (b, [1]), (c, [1]), (a, [3])], [2, 4])
    for fn in (a, b, c):
        ctx.fn_release(fn)                      # the trace keeps what it needs
    live0, bytes0 = ctx.stats()
    for rep in range(4):
        scale = np.float32(1 + rep)
        v = ctx.future_pending(pwb.PW_F32, (n,))
        y, z = prog.run([v], mode)
        assert ctx.future_query(y) == pwb.PW_ERR_NOT_READY and ctx.future_query(z) == pwb.PW_ERR_NOT_READY
        ctx.future_resolve(v, rows["input"] * scale)
        assert np.array_equal(ctx.await_(y), rows["input"] * scale * 2 + 1)
        assert np.array_equal(ctx.await_(z), rows["input"] * scale * 2 / 2 * 2)
        if rep == 0:
            assert np.array_equal(ctx.await_(y), rows["y"]) and np.array_equal(ctx.await_(z), rows["z"])
        for f in (v, y, z):
            ctx.future_release(f)
    assert ctx.stats() == (live0, bytes0)
    prog.close()


@pytest.mark.parametrize("mode", [pwb.PW_STREAM, pwb.PW_GRAPH])
def test_program_with_fan_in_and_two_inputs(ctx, orc, mode):
    """A diamond and a second input: s = (u + 1) + (u * 3); t = s + w; r = t / 2; returns (s, r).  s is both returned
    and consumed; intermediates are recycled inside the run."""
    n = 1000
    add1 = ctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, n, 1.0)
    mul3 = ctx.compile_scalar_fn(pwb.PW_FN_MUL_CONST, n, 3.0)
    half = ctx.compile_scalar_fn(pwb.PW_FN_DIV_CONST, n, 2.0)
    spec = pwb.make_spec(pwb.PW_F32, (n,))
    add2 = ctx.compile_fn(pwb.PW_FN_ADD2, [spec, spec], [spec])
    # values: 0 = u, 1 = w, 2 = u+1, 3 = u*3, 4 = s, 5 = t, 6 = r
    prog = pwb.Program(ctx, [spec, spec], [(add1, [0]), (mul3, [0]), (add2, [2, 3]), (add2, [4, 1]), (half, [5])], [4, 6])
    live0, bytes0 = ctx.stats()
    for rep in range(3):
        u = I.normal(5 + rep, 1, n, 1.0).astype(np.float32)
        w = I.normal(5 + rep, 2, n, 1.0).astype(np.float32)
        fu, fw = ctx.future_from_host(u), ctx.future_pending(pwb.PW_F32, (n,))
        s, r = prog.run([fu, fw], mode)
        ctx.future_resolve(fw, w)
        want_s = orc.scalar_fn("add", u, 1.0) + orc.scalar_fn("mul", u, 3.0)          # fp32 adds, rounded once each
        want_r = orc.scalar_fn("div", want_s + w, 2.0)
        assert np.array_equal(ctx.await_(s), want_s) and np.array_equal(ctx.await_(r), want_r)
        for f in (fu, fw, s, r):
            ctx.future_release(f)
    assert ctx.stats() == (live0, bytes0)
    prog.close()
    # a poisoned input poisons every output
    prog = pwb.Program(ctx, [spec, spec], [(add2, [0, 1]), (half, [2])], [3])
    fu, fw = ctx.future_from_host(np.zeros(n, np.float32)), ctx.future_pending(pwb.PW_F32, (n,))
    (r,) = prog.run([fu, fw], mode)
    ctx.future_resolve(fw, None)
    with pytest.raises(pwb.PwError) as e:
        ctx.await_(r)
    assert e.value.status == pwb.PW_ERR_POISONED
    for f in (fu, fw, r):
        ctx.future_release(f)
    prog.close()


def test_program_tracing_rejects_what_cannot_run(ctx):
    spec128, spec64 = pwb.make_spec(pwb.PW_F32, (128,)), pwb.make_spec(pwb.PW_F32, (64,))
    add128 = ctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, 128, 1.0)
    add64 = ctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, 64, 1.0)
    add2 = ctx.compile_fn(pwb.PW_FN_ADD2, [spec128, spec128], [spec128])
    with pytest.raises(pwb.PwError) as e:
        ctx.compile_fn(pwb.PW_FN_ADD2, [spec128, spec64], [spec128])
    assert e.value.status == pwb.PW_ERR_SHAPE
    for nodes, outs, status in [
        ([(add128, [0]), (add64, [1])], [2], pwb.PW_ERR_SHAPE),          # edge with the wrong shape
        ([(add128, [1])], [1], pwb.PW_ERR_INVALID),                      # reads a value defined later (itself)
        ([(add2, [0])], [1], pwb.PW_ERR_SHAPE),                          # wrong number of inputs
        ([(add128, [0])], [5], pwb.PW_ERR_INVALID),                      # returns a value that does not exist
        ([(add128, [0])], [0], pwb.PW_ERR_UNSUPPORTED),                  # returns its own input
    ]:
        with pytest.raises(pwb.PwError) as e:
            pwb.Program(ctx, [spec128], nodes, outs)
        assert e.value.status == status, (nodes, outs)
    prog = pwb.Program(ctx, [spec128], [(add128, [0])], [1])
    live0, bytes0 = ctx.stats()
    f64 = ctx.future_from_host(np.zeros(64, np.float32))
    with pytest.raises(pwb.PwError) as e:
        prog.run([f64])
    assert e.value.status == pwb.PW_ERR_SHAPE
    with pytest.raises(pwb.PwError):
        prog.run([f64, f64])
    ctx.future_release(f64)
    assert ctx.stats() == (live0, bytes0)
    prog.close()


# ---- object store: ownership labels, garbage collection, back-pressure (Section 4.6) ---------------------

def test_owner_labels_and_garbage_collection():
    ctx = pwb.Context(0)
    add1 = ctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, 128, 1.0)
    keep = ctx.future_from_host(np.zeros(128, np.float32))          # label 0
    live0, bytes0 = ctx.stats()
    ctx.set_owner(7)
    mine = [ctx.future_from_host(np.full(128, float(i), np.float32)) for i in range(3)]
    (derived,) = ctx.chain([add1] * 5, [mine[0]], 1, pwb.PW_STREAM)
    ctx.future_retain(derived)                                      # a second reference does not save it
    pending = ctx.future_pending(pwb.PW_F32, (128,))                # never resolved: its gate is cancelled
    ctx.set_owner(8)
    other = ctx.future_from_host(np.ones(128, np.float32))
    ctx.set_owner(0)
    assert ctx.stats()[0] == live0 + 6
    assert ctx.owner_collect(7) == 5
    assert ctx.stats()[0] == live0 + 1
    for h in mine + [derived, pending]:
        with pytest.raises(pwb.PwError):
            ctx.await_(h)                                           # the handles are dead
    assert np.array_equal(ctx.await_(other), np.ones(128, np.float32))   # other owners are untouched
    assert np.array_equal(ctx.await_(keep), np.zeros(128, np.float32))
    assert ctx.owner_collect(7) == 0
    assert ctx.owner_collect(8) == 1
    assert ctx.stats() == (live0, bytes0)
    ctx.close()


def test_memory_budget_refuses_direct_calls_and_stalls_scheduled_programs(orc):
    """Budget for three 1 MiB objects.  A direct call beyond it is refused with nothing enqueued; the scheduler
    stalls the programs instead and lets them through as the client collects earlier results."""
    n = 1 << 18                                                       # 1 MiB of fp32
    ctx = pwb.Context(0)
    add1 = ctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, n, 1.0)
    x = I.normal(9, 1, n, 1.0).astype(np.float32)
    f_in = ctx.future_from_host(x)
    base = ctx.stats()[1]
    ctx.set_memory_limit(base + 3 * (1 << 20) + 4096)
    held = [ctx.run_fn(add1, [f_in])[0] for _ in range(3)]
    live, used = ctx.stats()
    with pytest.raises(pwb.PwError) as e:
        ctx.run_fn(add1, [f_in])
    assert e.value.status == pwb.PW_ERR_OOM and ctx.stats() == (live, used)
    for h in held:
        ctx.future_release(h)
    # chains recycle their intermediates, so a long chain still fits
    (f,) = ctx.chain([add1] * 6, [f_in], 1, pwb.PW_STREAM)
    assert np.array_equal(ctx.await_(f), orc.chain_add(x, 6))
    ctx.future_release(f)
    sched = pwb.Scheduler(ctx, pwb.PW_SCHED_FIFO, max_in_flight=8)
    cid = sched.add_client(1.0)
    tickets = [sched.submit(cid, [add1] * (k + 1), f_in) for k in range(10)]   # ten results of 1 MiB: seven must wait
    time.sleep(0.05)
    programs, _, _ = sched.client_stats(cid)
    assert programs <= 4                                                # the rest is stalled, not failed
    for k, t in enumerate(tickets):
        assert np.array_equal(sched.wait(t, n), orc.chain_add(x, k + 1)), k
    stalled, ms = sched.stalls()
    assert stalled >= 1 and ms > 0
    sched.close()
    ctx.set_memory_limit(0)
    ctx.close()


def test_failed_client_is_garbage_collected_and_the_others_carry_on(orc):
    ctx = pwb.Context(0)
    sched = pwb.Scheduler(ctx, pwb.PW_SCHED_FIFO, max_in_flight=2)
    busy = ctx.compile_scalar_fn(pwb.PW_FN_BUSY, 128, 1.0, busy_us=300.0)
    add1 = ctx.compile_scalar_fn(pwb.PW_FN_ADD_CONST, 128, 1.0)
    x = I.dispatch_input()
    f_in = ctx.future_from_host(x)
    live0, bytes0 = ctx.stats()
    good, bad = sched.add_client(1.0), sched.add_client(1.0)
    done_bad = [sched.submit(bad, [add1], f_in) for _ in range(3)]
    sched.drain()                                                       # three results sit uncollected
    queued_bad = [sched.submit(bad, [busy] * 8, f_in) for _ in range(6)]
    t_good = sched.submit(good, [add1] * 4, f_in)
    released = sched.client_fail(bad)
    assert released >= 3
    for t in done_bad + queued_bad[3:]:                                 # (the first ones may already have been handed out)
        with pytest.raises(pwb.PwError) as e:
            sched.wait(t)
        assert e.value.status == pwb.PW_ERR_POISONED
    with pytest.raises(pwb.PwError):
        sched.submit(bad, [add1], f_in)
    assert np.array_equal(sched.wait(t_good, 128), orc.chain_add(x, 4))
    sched.close()
    assert ctx.stats() == (live0, bytes0)
    ctx.close()
