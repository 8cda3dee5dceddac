"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle cannot run the 12-layer workload whole, so each kernel is run at its full cfg3 shape and a
sample of its outputs is recomputed one by one by the oracle from the very operands the kernel read
(copied back from the GPU); the whole step is checked through properties that hold at any size."""
import math

import numpy as np
import pytest
import torch

from paper_2203_12533_amd import binding as pwb
from paper_2203_12533_amd import inputs as I
from gpu_util import assert_close, dev_f32, dev_i32, host, ptr, rel_l2

pytestmark = pytest.mark.gpu
CFG3 = I.workload("cfg3")
N, D, F, V, T, H = CFG3.n_tokens, CFG3.d_model, CFG3.d_ff, CFG3.vocab, CFG3.seq, CFG3.n_head


@pytest.fixture(scope="module")
def ctx():
    c = pwb.Context(0)
    yield c
    c.close()


def _bf16_randn(shape, seed, std=1.0):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    return (torch.randn(shape, device="cuda", generator=g) * std).to(torch.bfloat16)


ROWS = np.array([0, 1, 255, 256, 4097, 8191])


@pytest.mark.parametrize("name,n_out,k_in", [("qkv", 3 * D, D), ("ffn1", F, D), ("ffn2", D, F), ("head", V, D)])
def test_forward_gemms_at_cfg3_shape(ctx, orc, name, n_out, k_in):
    x, w = _bf16_randn((N, k_in), 1), _bf16_randn((k_in, n_out), 2, 0.02)
    out = torch.empty((N, n_out), dtype=torch.bfloat16, device="cuda")
    ctx.gemm(dtype=pwb.PW_BF16, a_kmajor=0, b_kmajor=1, M=N, N=n_out, K=k_in, lda=k_in, ldb=n_out, ldc=n_out,
             epilogue=pwb.PW_EPI_STORE, out_dtype=pwb.PW_BF16, accumulate=0, A=ptr(x), B=ptr(w), C=ptr(out))
    ctx.synchronize()
    ref = orc.linear_fwd(host(x[ROWS]), host(w))
    assert_close(host(out[ROWS]), ref, 4e-3)


def test_gemms_of_a_pipeline_stage_micro_batch_at_cfg4_shape(ctx, orc):
    """cfg4's micro-batches of 2048 tokens give the GEMMs that write d_model = 4096 columns only 128 full tiles;
    they run on 128 x 256 tiles.  FFN2 forward (K = 16384) with the residual epilogue and the FFN1 data gradient
    (both operands k-contiguous) at full shape, sampled rows against the oracle."""
    c4 = I.workload("cfg4")
    n, d, f = c4.n_tokens, c4.d_model, c4.d_ff
    assert (n // 256) * (d // 256) == 128
    rows = np.array([0, 127, 128, 255, 256, 1029, n - 1])
    h, w2 = _bf16_randn((n, f), 11), _bf16_randn((f, d), 12, 0.02)
    g = torch.Generator(device="cuda")
    g.manual_seed(13)
    res = torch.randn((n, d), device="cuda", generator=g)
    bias = torch.randn((d,), device="cuda", generator=g)
    out = torch.empty((n, d), dtype=torch.float32, device="cuda")
    ctx.gemm(dtype=pwb.PW_BF16, a_kmajor=0, b_kmajor=1, M=n, N=d, K=f, lda=f, ldb=d, ldc=d,
             epilogue=pwb.PW_EPI_BIAS_RESIDUAL, out_dtype=pwb.PW_F32, accumulate=0, A=ptr(h), B=ptr(w2), bias=ptr(bias),
             aux=ptr(res), C=ptr(out))
    du, w1 = _bf16_randn((n, f), 14), _bf16_randn((d, f), 15, 0.02)
    dx = torch.empty((n, d), dtype=torch.bfloat16, device="cuda")
    ctx.gemm(dtype=pwb.PW_BF16, a_kmajor=0, b_kmajor=0, M=n, N=d, K=f, lda=f, ldb=f, ldc=d,
             epilogue=pwb.PW_EPI_STORE, out_dtype=pwb.PW_BF16, accumulate=0, A=ptr(du), B=ptr(w1), C=ptr(dx))
    ctx.synchronize()
    ref = orc.linear_fwd(host(h[rows]), host(w2), host(bias).astype(np.float64)) + host(res[rows])
    assert_close(host(out[rows]), ref, 1e-5)
    rdx, _, _ = orc.linear_bwd(np.zeros((len(rows), d)), host(w1), host(du[rows]))
    assert_close(host(dx[rows]), rdx, 4e-3)


@pytest.mark.parametrize("name,n_in,k_out", [("ffn2", F, D), ("ffn1", D, F), ("head", D, V)])
def test_dgrad_and_wgrad_gemms_at_cfg3_shape(ctx, orc, name, n_in, k_out):
    dy, w, x = _bf16_randn((N, k_out), 3), _bf16_randn((n_in, k_out), 4, 0.02), _bf16_randn((N, n_in), 5)
    dx = torch.empty((N, n_in), dtype=torch.bfloat16, device="cuda")
    ctx.gemm(dtype=pwb.PW_BF16, a_kmajor=0, b_kmajor=0, M=N, N=n_in, K=k_out, lda=k_out, ldb=k_out, ldc=n_in,
             epilogue=pwb.PW_EPI_STORE, out_dtype=pwb.PW_BF16, accumulate=0, A=ptr(dy), B=ptr(w), C=ptr(dx))
    dw = torch.empty((n_in, k_out), dtype=torch.float32, device="cuda")
    ctx.gemm(dtype=pwb.PW_BF16, a_kmajor=1, b_kmajor=1, M=n_in, N=k_out, K=N, lda=n_in, ldb=k_out, ldc=k_out,
             epilogue=pwb.PW_EPI_STORE, out_dtype=pwb.PW_F32, accumulate=0, A=ptr(x), B=ptr(dy), C=ptr(dw))
    ctx.synchronize()
    rdx, _, _ = orc.linear_bwd(np.zeros((len(ROWS), n_in)), host(w), host(dy[ROWS]))
    assert_close(host(dx[ROWS]), rdx, 4e-3)
    cols = np.array([0, 7, 255, 256, n_in - 1])                 # sampled input features = rows of dW
    _, rdw, _ = orc.linear_bwd(host(x[:, cols]), np.zeros((len(cols), k_out)), host(dy))
    assert_close(host(dw[cols]), rdw, 1e-5)


def test_paired_attention_weight_gradients_at_cfg3_shape(ctx, orc):
    """dWqkv = a^T . dqkv and dWo = o^T . dy in one launch (192 + 64 tiles = one workgroup per compute unit),
    against the oracle on sampled rows, and in agreement with the two single launches everywhere (the single
    out-projection launch takes another tile shape, so its summation order differs)."""
    a, dqkv = _bf16_randn((N, D), 11), _bf16_randn((N, 3 * D), 12)
    o, dy = _bf16_randn((N, D), 13), _bf16_randn((N, D), 14)
    def args(x, g, out, n_out):
        return dict(dtype=pwb.PW_BF16, a_kmajor=1, b_kmajor=1, M=D, N=n_out, K=N, lda=D, ldb=n_out, ldc=n_out,
                    epilogue=pwb.PW_EPI_STORE, out_dtype=pwb.PW_F32, accumulate=0, A=ptr(x), B=ptr(g), C=ptr(out))
    dwqkv = torch.full((D, 3 * D), float("nan"), device="cuda")
    dwo = torch.full((D, D), float("nan"), device="cuda")
    dbqkv = torch.full((3 * D,), float("nan"), device="cuda")      # the bias gradient rides along: column sums of dqkv
    ctx.gemm_pair({**args(a, dqkv, dwqkv, 3 * D), "b_colsum": ptr(dbqkv)}, args(o, dy, dwo, D))
    one_qkv, one_o = torch.empty_like(dwqkv), torch.empty_like(dwo)
    ctx.gemm(**args(a, dqkv, one_qkv, 3 * D))
    ctx.gemm(**args(o, dy, one_o, D))
    ctx.synchronize()
    cols = np.array([0, 9, 255, 256, 1031, D - 1])
    _, want, _ = orc.linear_bwd(host(a[:, cols]), np.zeros((len(cols), 3 * D)), host(dqkv))
    assert_close(host(dwqkv[cols]), want, 1e-5)
    _, want, _ = orc.linear_bwd(host(o[:, cols]), np.zeros((len(cols), D)), host(dy))
    assert_close(host(dwo[cols]), want, 1e-5)
    assert_close(host(one_o[cols]), want, 1e-5)
    assert_close(host(dbqkv), host(dqkv).astype(np.float64).sum(axis=0), 1e-5)
    # alone (192 tiles: the ring kernel) and accumulating into what is there
    acc_w, acc_b = torch.ones_like(dwqkv), torch.ones_like(dbqkv)
    ctx.gemm(**{**args(a, dqkv, acc_w, 3 * D), "accumulate": 1, "b_colsum": ptr(acc_b)})
    ctx.synchronize()
    assert_close(host(acc_b), host(dqkv).astype(np.float64).sum(axis=0) + 1.0, 1e-5)
    assert_close(host(acc_w), host(one_qkv) + 1.0, 1e-6)
    with pytest.raises(pwb.PwError):                               # 64 tiles alone: not served, nothing launched
        ctx.gemm(**{**args(o, dy, dwo, D), "b_colsum": ptr(acc_b)})
    assert torch.isfinite(dwqkv).all() and torch.isfinite(dwo).all()
    assert_close(host(dwqkv), host(one_qkv), 1e-6)
    assert_close(host(dwo), host(one_o), 1e-6)


@pytest.mark.parametrize("workload,problems", [("cfg3", [(0, 0), (3, 7), (7, 15)]), ("cfg4", [(0, 0), (0, 31)]),
                                               ("cfg5", [(0, 5), (1, 63)])])
def test_attention_at_full_shapes(ctx, orc, workload, problems):
    """Causal attention at the batch / sequence / head counts of the measured workloads (8 x 1024 x 16,
    1 x 2048 x 32, 2 x 2048 x 64; the number of 128-row blocks per problem decides how the blocks of several
    problems are interleaved), a few (batch, head) problems recomputed whole by the oracle."""
    cfg = I.workload(workload)
    B, hd, T, H = cfg.batch, cfg.head_dim, cfg.seq, cfg.n_head
    N, D = B * T, H * hd
    qkv = _bf16_randn((N, 3 * D), 6)
    o = torch.empty((N, D), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((B, H, T), device="cuda")
    ctx.op("attention_fwd", pwb.PW_BF16, ptr(qkv), ptr(o), ptr(lse), B, T, H, hd)
    dout = _bf16_randn((N, D), 7)
    dqkv = torch.empty((N, 3 * D), dtype=torch.bfloat16, device="cuda")
    delta = torch.empty((B, H, T), device="cuda")
    ctx.op("attention_bwd", pwb.PW_BF16, ptr(qkv), ptr(o), ptr(dout), ptr(lse), ptr(delta), ptr(dqkv), B, T, H, hd)
    ctx.synchronize()
    for (b, h) in problems:                                       # sampled (batch, head) problems, recomputed whole
        rows = slice(b * T, (b + 1) * T)
        cols = [slice(p * D + h * hd, p * D + (h + 1) * hd) for p in range(3)]
        sub = np.concatenate([host(qkv[rows, c]) for c in cols], axis=1)       # a 1-batch, 1-head problem
        ro = orc.attention_fwd(sub, 1, T, 1, hd)
        assert_close(host(o[rows, cols[0]]), ro, 6e-3, (b, h))
        rd = orc.attention_bwd(sub, host(dout[rows, cols[0]]), 1, T, 1, hd)
        got = np.concatenate([host(dqkv[rows, c]) for c in cols], axis=1)
        for p in range(3):
            assert_close(got[:, p * hd:(p + 1) * hd], rd[:, p * hd:(p + 1) * hd], 1.5e-2, (b, h, p))


def test_layernorm_and_xent_at_cfg3_shape(ctx, orc):
    x = torch.randn((N, D), device="cuda") * 2 + 0.3
    g, b = dev_f32(1 + 0.1 * I.normal(1, 1, D)), dev_f32(0.1 * I.normal(1, 2, D))
    y = torch.empty((N, D), dtype=torch.bfloat16, device="cuda")
    mean, rstd = torch.empty(N, device="cuda"), torch.empty(N, device="cuda")
    ctx.op("layernorm_fwd", pwb.PW_BF16, ptr(x), ptr(g), ptr(b), ptr(y), ptr(mean), ptr(rstd), N, D)
    ctx.synchronize()
    ry, rmean, rrstd = orc.layernorm_fwd(host(x[ROWS]), host(g), host(b))
    assert_close(host(y[ROWS]), ry, 4e-3)
    assert_close(host(mean[ROWS]), rmean, 1e-5)
    assert_close(host(rstd[ROWS]), rrstd, 1e-5)
    # backward in the step's configuration: bf16 dy, fp32 residual gradient in, fp32 + bf16 dx out, column sums
    dy, dres = _bf16_randn((N, D), 21), torch.randn((N, D), device="cuda")
    dx, dxlp = torch.empty((N, D), device="cuda"), torch.empty((N, D), dtype=torch.bfloat16, device="cuda")
    dg, db, dsum = (torch.empty(D, device="cuda") for _ in range(3))
    ws = torch.empty(pwb.lib().pw_layernorm_bwd_ws_floats(N, D), device="cuda")
    ctx.op("layernorm_bwd", pwb.PW_BF16, ptr(dy), ptr(x), ptr(g), ptr(mean), ptr(rstd), ptr(dres), ptr(dx), ptr(dxlp),
           ptr(dg), ptr(db), ptr(dsum), ptr(ws), N, D, 0)
    ctx.synchronize()
    rdx, rdg, rdb = orc.layernorm_bwd(host(dy), host(x), host(g))        # the whole tensor: 16.8 M elements
    want = rdx + host(dres)
    assert_close(host(dx), want, 1e-5)
    assert_close(host(dxlp), want, 4e-3)
    assert_close(host(dg), rdg, 1e-5)
    assert_close(host(db), rdb, 1e-5)
    assert_close(host(dsum), want.sum(axis=0), 1e-5)
    z = _bf16_randn((N, V), 8, 1.5)
    tok = I.lm_tokens(CFG3)
    tokd = dev_i32(tok)
    keep = host(z[ROWS])
    loss, rows = torch.empty(1, device="cuda"), torch.empty(N, device="cuda")
    ctx.op("softmax_xent", pwb.PW_BF16, ptr(z), ptr(tokd), ptr(loss), ptr(rows), CFG3.batch, T, V)
    ctx.synchronize()
    tgt = tok[:, 1:].reshape(-1)
    for i, r in enumerate(ROWS):
        rl, rdz = orc.softmax_xent(keep[i:i + 1], tgt[r:r + 1])
        assert abs(host(rows)[r] - rl) / rl < 1e-5
        assert_close(host(z[r]) * N, rdz[0], 6e-3)              # the kernel divides by the full N
    assert abs(host(loss)[0] - host(rows).mean()) < 1e-5


def test_full_cfg3_step_properties():
    """Whole 12-layer step: finite loss near ln V + sigma^2/2 at initialisation, loss falls over steps on a
    fixed batch, and two identically seeded runs agree bit for bit."""
    def run():
        with pwb.Context(0) as ctx:
            model = ctx.model(CFG3)
            for name, shape, kind in I.param_shapes(CFG3):      # the workload's seeded weights, drawn on the GPU
                t = I.param_torch(CFG3, name, shape, kind, "cuda")
                torch.cuda.synchronize()
                model.import_device(pwb.PW_PARAMS, name, t.data_ptr())
            step = model.compile_train_step()
            ft = ctx.future_from_host(I.lm_tokens(CFG3))
            losses = []
            for _ in range(3):
                fl = ctx.train_step(step, ft)
                losses.append(float(ctx.await_(fl)[0]))
                ctx.future_release(fl)
            gsum = model.export(pwb.PW_GRADS, "l11.w2")
            wte = model.export(pwb.PW_GRADS, "wte")
            model.close()
            return losses, gsum, wte
    l1, g1, e1 = run()
    l2, g2, e2 = run()
    assert all(math.isfinite(v) for v in l1)
    # logits are ~N(0, 0.02^2 * 2048) = N(0, 0.82): E[loss] = ln V + 0.82/2 within sampling noise
    assert abs(l1[0] - (math.log(V) + 0.41)) < 0.1, l1
    assert l1[2] < l1[1] < l1[0]
    assert l1 == l2 and np.array_equal(g1, g2) and np.array_equal(e1, e2)
    used = np.unique(I.lm_tokens(CFG3)[:, :-1])
    unused = np.setdiff1d(np.arange(V), used)[:50]
    assert (e1.reshape(V, D)[unused] == 0).all() and np.abs(e1.reshape(V, D)[used[:50]]).max() > 0


def test_three_weight_gradients_share_one_launch(ctx, orc):
    """The weight gradients of a decoder's attention over the encoder output at the encoder-decoder workload's
    shape - dWkv = mem^T . dkv (128 tiles), dWq = a^T . dq and dWox = o^T . dy (64 tiles each) - in one launch
    of 256 workgroups, with the two bias gradients riding along: against the oracle on sampled rows and against
    single launches everywhere."""
    mem, dkv = _bf16_randn((N, D), 21), _bf16_randn((N, 2 * D), 22)
    a, dq = _bf16_randn((N // 2, D), 23), _bf16_randn((N // 2, D), 24)      # fewer target than source positions
    o, dy = _bf16_randn((N // 2, D), 25), _bf16_randn((N // 2, D), 26)
    def args(x, g, out, n_out):
        return dict(dtype=pwb.PW_BF16, a_kmajor=1, b_kmajor=1, M=D, N=n_out, K=x.shape[0], lda=D, ldb=n_out, ldc=n_out,
                    epilogue=pwb.PW_EPI_STORE, out_dtype=pwb.PW_F32, accumulate=0, A=ptr(x), B=ptr(g), C=ptr(out))
    nan = float("nan")
    dwkv, dwq, dwox = (torch.full(s, nan, device="cuda") for s in ((D, 2 * D), (D, D), (D, D)))
    dbkv, dbq = torch.full((2 * D,), nan, device="cuda"), torch.full((D,), nan, device="cuda")
    ctx.gemm_group([{**args(a, dq, dwq, D), "b_colsum": ptr(dbq)}, {**args(mem, dkv, dwkv, 2 * D), "b_colsum": ptr(dbkv)},
                    args(o, dy, dwox, D)])
    singles = [torch.empty_like(t) for t in (dwkv, dwq, dwox)]
    for (x, g, n_out), out in zip(((mem, dkv, 2 * D), (a, dq, D), (o, dy, D)), singles):
        ctx.gemm(**args(x, g, out, n_out))
    ctx.synchronize()
    cols = np.array([0, 9, 255, 256, 1031, D - 1])
    for x, g, got in ((mem, dkv, dwkv), (a, dq, dwq), (o, dy, dwox)):
        _, want, _ = orc.linear_bwd(host(x[:, cols]), np.zeros((len(cols), g.shape[1])), host(g))
        assert_close(host(got[cols]), want, 1e-5)
    assert_close(host(dbkv), host(dkv).astype(np.float64).sum(axis=0), 1e-5)
    assert_close(host(dbq), host(dq).astype(np.float64).sum(axis=0), 1e-5)
    for got, one in zip((dwkv, dwq, dwox), singles):
        assert_close(host(got), host(one), 1e-6)
    with pytest.raises(pwb.PwError):                               # a bad member: nothing is launched
        ctx.gemm_group([args(a, dq, dwq, D), {**args(mem, dkv, dwkv, 2 * D), "ldb": 8}, args(o, dy, dwox, D)])


@pytest.fixture(scope="module")
def one_layer(orc):
    """One layer with cfg3's d_model / heads / FFN width and full sequence length, 2048 tokens, vocabulary cut to 8192
    (the oracle's step then takes about 20 s): parameters, tokens and the oracle's first TWO steps."""
    cfg = CFG3.with_(n_layer=1, batch=2, vocab=8192)
    tok = I.lm_tokens(cfg)
    rng = np.random.default_rng(20)            # 84 M parameters: numpy's generator draws them in a second
    params = {}
    for name, shape, kind in I.param_shapes(cfg):
        a = rng.standard_normal(int(np.prod(shape)), dtype=np.float32) * np.float32(cfg.init_std)
        if kind == "gain":
            a += np.float32(1.0)
        params[name] = I.round_to_bf16(a).reshape(shape)       # biases and gains perturbed too
    ref1 = orc.lm_train_step(cfg, params, tok)
    ref2 = orc.lm_train_step(cfg, ref1["params"], tok, state={"m": ref1["m"], "v": ref1["v"]}, t=2, backward=False, update=False)
    return cfg, params, tok, ref1, ref2["loss"]


def test_one_layer_step_at_cfg3_layer_shapes_matches_oracle(one_layer):
    """The production kernels end to end against the oracle: the forward, data-gradient and weight-gradient GEMMs all
    run on the ring-buffered kernel (192-1024 tiles), the weight-gradient pair and the fused bias-gradient sums
    included, the head_dim-128 attention kernels see 1024-token sequences and LayerNorm its one-wave-per-row path.
    Loss and every gradient tensor are compared."""
    cfg, params, tok, ref, _ = one_layer
    with pwb.Context(0) as ctx:
        model = ctx.model(cfg)
        model.load_params(params)
        step = model.compile_train_step()
        ft = ctx.future_from_host(tok)
        fl = ctx.train_step(step, ft)
        loss = float(ctx.await_(fl)[0])
        assert abs(loss - ref["loss"]) / abs(ref["loss"]) < 2e-2, (loss, ref["loss"])
        grads = model.export_all(pwb.PW_GRADS, params)
        worst = ("", 0.0)
        for k, g in grads.items():
            err = rel_l2(g, ref["grads"][k])
            worst = max(worst, (k, err), key=lambda t: t[1])
            assert_close(g, ref["grads"][k], 2e-2, k)
        print("worst gradient error", worst)
        model.close()


@pytest.mark.parametrize("fused_update,fused_head_loss", [(True, False), (False, True), (True, True)])
def test_one_layer_step_with_fused_update_and_fused_head_loss(one_layer, fused_update, fused_head_loss):
    """The same step with Adam inside the weight-gradient epilogues and / or the LM head fused with the loss.  The
    gradients of the fused weights are never stored; after the first step Adam's first moment is (1 - beta1) g, so
    m / (1 - beta1) is compared with the oracle's gradient element by element, v with (1 - beta2) g^2, the bf16 copy
    with the master weights; the other gradients are read as usual; the loss of the SECOND step (which sees the
    updated weights) must follow the oracle's.  Twice, stream and HIP-graph dispatch: same bits."""
    cfg, params, tok, ref, ref_loss2 = one_layer
    big = [k for k in params if k.split(".")[-1] in ("wqkv", "wo", "w1", "w2", "wh")]
    results = []
    for mode in (pwb.PW_STREAM, pwb.PW_GRAPH):
        with pwb.Context(0) as ctx:
            model = ctx.model(cfg, fused_update=fused_update, fused_head_loss=fused_head_loss)
            model.load_params(params)
            step = model.compile_train_step()
            ft = ctx.future_from_host(tok)
            losses = []
            for it in range(2):
                (fl,) = ctx.chain([step], [ft], 1, mode)
                losses.append(float(ctx.await_(fl)[0]))
                ctx.future_release(fl)
                if it == 0 and mode == pwb.PW_STREAM:
                    assert abs(losses[0] - ref["loss"]) / abs(ref["loss"]) < 2e-2, (losses, ref["loss"])
                    new1 = model.export_all(pwb.PW_PARAMS, params)
                    m1 = model.export_all(pwb.PW_ADAM_M, params)
                    v1 = model.export_all(pwb.PW_ADAM_V, params)
                    for k in params:
                        g_ref = ref["grads"][k]
                        assert_close(m1[k].astype(np.float64) / (1 - cfg.beta1), g_ref, 2e-2, k + " (from m)")
                        assert_close(v1[k].astype(np.float64) / (1 - cfg.beta2), g_ref ** 2, 4e-2, k + " (from v)")
                        if fused_update and k in big:
                            with pytest.raises(pwb.PwError) as e:
                                model.export(pwb.PW_GRADS, k)
                            assert e.value.status == pwb.PW_ERR_UNSUPPORTED
                        else:
                            assert_close(model.export(pwb.PW_GRADS, k).reshape(g_ref.shape), g_ref, 2e-2, k)
            # the second step saw the weights the first one wrote (master copy and bf16 copy alike)
            assert abs(losses[1] - ref_loss2) / abs(ref_loss2) < 2e-2, (losses, ref_loss2)
            assert losses[1] < losses[0]
            results.append((losses, model.export_all(pwb.PW_PARAMS, params), model.export_all(pwb.PW_ADAM_V, params)))
            model.close()
    assert results[0][0] == results[1][0]
    for k in params:
        assert np.array_equal(results[0][1][k], results[1][1][k]), k
        assert np.array_equal(results[0][2][k], results[1][2][k]), k
    # Adam's first update is -lr sign(g) wherever |g| >> eps: the updated weights are compared through that
    for k in big:
        g_ref = ref["grads"][k].reshape(-1)
        sure = np.abs(g_ref) > 0.05 * np.sqrt(np.mean(g_ref ** 2))        # the sign of g is beyond the bf16 error there
        moved = (new1[k].astype(np.float64) - params[k].astype(np.float64)).reshape(-1)[sure]
        assert (np.sign(moved) == -np.sign(g_ref[sure])).mean() > 0.999, k


def test_one_layer_step_at_cfg5_width_matches_oracle(orc):
    """The wide-layer workload's width end to end against the oracle: one layer with d_model 8192 and 64 heads of 128
    (LayerNorm's block-per-row path, contraction length 8192 in the ring-buffered GEMM, 3072-tile weight gradients,
    the 128 x 256-tile kernel for the out-projection), 2 x 256 tokens; FFN width and vocabulary are cut (4096, 2048)
    so that the fp64 oracle's 0.37 G parameters fit the host and its step takes tens of seconds.  Loss and every
    gradient tensor are compared, weights drawn with the workload's own standard deviation."""
    c5 = I.workload("cfg5")
    cfg = c5.with_(n_layer=1, batch=2, seq=256, d_ff=4096, vocab=2048)
    assert cfg.d_model == 8192 and cfg.n_head == 64 and cfg.head_dim == 128
    tok = I.lm_tokens(cfg)
    rng = np.random.default_rng(22)
    params = {}
    for name, shape, kind in I.param_shapes(cfg):
        a = rng.standard_normal(int(np.prod(shape)), dtype=np.float32) * np.float32(cfg.init_std)
        if kind == "gain":
            a += np.float32(1.0)
        params[name] = I.round_to_bf16(a).reshape(shape)       # biases and gains perturbed too
    ref = orc.lm_train_step(cfg, params, tok, update=False)
    with pwb.Context(0) as ctx:
        model = ctx.model(cfg)
        model.load_params(params)
        step = model.compile_train_step()
        ft = ctx.future_from_host(tok)
        fl = ctx.train_step(step, ft)
        loss = float(ctx.await_(fl)[0])
        assert abs(loss - ref["loss"]) / abs(ref["loss"]) < 2e-2, (loss, ref["loss"])
        worst = ("", 0.0)
        for k in params:
            g = model.export(pwb.PW_GRADS, k).reshape(ref["grads"][k].shape)
            worst = max(worst, (k, rel_l2(g, ref["grads"][k])), key=lambda t: t[1])
            assert_close(g, ref["grads"][k], 2e-2, k)
        print("worst gradient error", worst)
        model.close()


@pytest.mark.parametrize("name,n_out,k_in", [("qkv", 3 * 8192, 8192), ("ffn1", 32768, 8192), ("ffn2", 8192, 32768)])
def test_gemms_at_cfg5_shape(ctx, orc, name, n_out, k_in):
    """Forward, data-gradient and weight-gradient GEMMs at the wide-layer workload's shapes (4096 tokens; contraction
    and leading dimensions of 8192 and 32768), sampled rows of each product recomputed by the oracle from the very
    operands the kernel read."""
    n = I.workload("cfg5").n_tokens
    x, w = _bf16_randn((n, k_in), 31), _bf16_randn((k_in, n_out), 32, 0.01)
    out = torch.empty((n, n_out), dtype=torch.bfloat16, device="cuda")
    ctx.gemm(dtype=pwb.PW_BF16, a_kmajor=0, b_kmajor=1, M=n, N=n_out, K=k_in, lda=k_in, ldb=n_out, ldc=n_out,
             epilogue=pwb.PW_EPI_STORE, out_dtype=pwb.PW_BF16, accumulate=0, A=ptr(x), B=ptr(w), C=ptr(out))
    dy = _bf16_randn((n, n_out), 33)
    dx = torch.empty((n, k_in), dtype=torch.bfloat16, device="cuda")
    ctx.gemm(dtype=pwb.PW_BF16, a_kmajor=0, b_kmajor=0, M=n, N=k_in, K=n_out, lda=n_out, ldb=n_out, ldc=k_in,
             epilogue=pwb.PW_EPI_STORE, out_dtype=pwb.PW_BF16, accumulate=0, A=ptr(dy), B=ptr(w), C=ptr(dx))
    dw = torch.empty((k_in, n_out), dtype=torch.float32, device="cuda")
    ctx.gemm(dtype=pwb.PW_BF16, a_kmajor=1, b_kmajor=1, M=k_in, N=n_out, K=n, lda=k_in, ldb=n_out, ldc=n_out,
             epilogue=pwb.PW_EPI_STORE, out_dtype=pwb.PW_F32, accumulate=0, A=ptr(x), B=ptr(dy), C=ptr(dw))
    ctx.synchronize()
    rows = np.array([0, 255, 256, 2049, n - 1])
    wh = host(w)
    assert_close(host(out[rows]), orc.linear_fwd(host(x[rows]), wh), 4e-3, "forward")
    rdx, _, _ = orc.linear_bwd(np.zeros((len(rows), k_in)), wh, host(dy[rows]))
    assert_close(host(dx[rows]), rdx, 4e-3, "data gradient")
    del wh
    cols = np.array([0, 7, 256, k_in - 1])                       # sampled input features = rows of dW
    _, rdw, _ = orc.linear_bwd(host(x[:, cols]), np.zeros((len(cols), n_out)), host(dy))
    assert_close(host(dw[cols]), rdw, 1e-5, "weight gradient")


def test_one_layer_encoder_decoder_step_at_full_layer_width_matches_oracle(orc):
    """The encoder-decoder step end to end at the width of the measured workload: one encoder and one decoder layer
    with d_model 2048 / 16 heads / FFN 8192, 2 x 1024 source and 2 x 512 target positions, so that the ring-buffered
    GEMM kernel, the three-way weight-gradient launch of the cross-attention sub-block with its fused bias
    gradients, the fp32-accumulating data-gradient GEMM into the encoder output's gradient and the head_dim-128
    attention kernels in their three roles (unmasked 1024 x 1024, causal 512 x 512, 512 queries over 1024 keys) all
    run on real shapes.  Loss and every gradient tensor are compared (vocabulary cut to 8192 for the oracle's sake)."""
    cfg = I.EncDecConfig(1, 1, D, H, F, 8192, 1024, 512, 2, bf16=True, optimizer="adam", lr=1e-4)
    src, tgt = I.encdec_tokens(cfg)
    rng = np.random.default_rng(21)
    params = {}
    for name, shape, kind in I.encdec_param_shapes(cfg):
        a = rng.standard_normal(int(np.prod(shape)), dtype=np.float32) * np.float32(cfg.init_std)
        if kind == "gain":
            a += np.float32(1.0)
        params[name] = I.round_to_bf16(a).reshape(shape)       # biases and gains perturbed too
    ref = orc.encdec_train_step(cfg, params, src, tgt)
    with pwb.Context(0) as ctx:
        model = ctx.encdec(cfg)
        model.load_params(params)
        step = model.compile_train_step()
        fs, ft = ctx.future_from_host(src), ctx.future_from_host(tgt)
        (fl,) = ctx.run_fn(step, [fs, ft], 1)
        loss = float(ctx.await_(fl)[0])
        assert abs(loss - ref["loss"]) / abs(ref["loss"]) < 2e-2, (loss, ref["loss"])
        grads = model.export_all(pwb.PW_GRADS, params)
        worst = ("", 0.0)
        for k, g in grads.items():
            err = rel_l2(g, ref["grads"][k])
            worst = max(worst, (k, err), key=lambda t: t[1])
            assert_close(g, ref["grads"][k], 2e-2, k)
        print("worst gradient error", worst)
        plain = model.export_all(pwb.PW_PARAMS, params)            # after the step's Adam launch
        model.close()
    # The same step with every GEMM weight updated inside its weight-gradient GEMM (the pair, the three-way launch and
    # the single launches alike).  Those gradients are not stored: after the first step m / (1 - beta1) is the
    # gradient and v / (1 - beta2) its square; the update itself must be the one the optimizer launch made above from
    # the same accumulator values.
    big = [k for k in params if k.split(".")[-1] in ("wqkv", "wo", "wq", "wkv", "wox", "w1", "w2", "wh")]
    assert len(big) == 12
    with pwb.Context(0) as ctx:
        model = ctx.encdec(cfg, fused_update=True)
        model.load_params(params)
        step = model.compile_train_step()
        fs, ft = ctx.future_from_host(src), ctx.future_from_host(tgt)
        (fl,) = ctx.run_fn(step, [fs, ft], 1)
        loss = float(ctx.await_(fl)[0])
        assert abs(loss - ref["loss"]) / abs(ref["loss"]) < 2e-2, (loss, ref["loss"])
        m1 = model.export_all(pwb.PW_ADAM_M, params)
        v1 = model.export_all(pwb.PW_ADAM_V, params)
        new = model.export_all(pwb.PW_PARAMS, params)
        for k in params:
            g_ref = ref["grads"][k]
            assert_close(m1[k].astype(np.float64).reshape(g_ref.shape) / (1 - cfg.beta1), g_ref, 2e-2, k + " (from m)")
            assert_close(v1[k].astype(np.float64).reshape(g_ref.shape) / (1 - cfg.beta2), g_ref ** 2, 4e-2, k + " (from v)")
            if k in big:
                with pytest.raises(pwb.PwError) as e:
                    model.export(pwb.PW_GRADS, k)
                assert e.value.status == pwb.PW_ERR_UNSUPPORTED
            else:
                assert_close(model.export(pwb.PW_GRADS, k).reshape(g_ref.shape), g_ref, 2e-2, k)
            w0 = params[k].astype(np.float64).reshape(-1)
            assert_close(new[k].astype(np.float64).reshape(-1) - w0, plain[k].astype(np.float64).reshape(-1) - w0, 1e-4,
                         k + " (update)", extra=np.abs(w0) * 1.2e-7)
        # a second step runs on the weights and bf16 copies the epilogues wrote
        (fl2,) = ctx.run_fn(step, [fs, ft], 1)
        loss2 = float(ctx.await_(fl2)[0])
        assert loss2 < loss
        model.close()
