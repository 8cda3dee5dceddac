"""Per-kernel parity: every HIP kernel, called through the C boundary, against the CPU oracle on the same
seeded inputs.  Sizes span several tiles and ragged tails.  Bars (relative L2 per tensor): fp32 path 1e-4,
bf16 path 2e-2; where the arithmetic allows a much tighter bound the test uses it."""
import numpy as np
import pytest
import torch

from paper_2203_12533_amd import binding as pwb
from paper_2203_12533_amd import inputs as I
from gpu_util import DT, TOL, assert_close, dev_act, dev_f32, dev_i32, empty_act, host, ptr, rel_l2

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = pwb.Context(0)
    yield c
    c.close()


def _rand(seed, shape, std=1.0):
    return I.normal(seed, 77, int(np.prod(shape)), std).reshape(shape)


# ---- GEMM ---------------------------------------------------------------------------------------------

# (4096, 4096, K): 256 full 256x256 tiles, the ring-buffered kernel, with 1, 2 and 3 k-tiles of 64;
# (1024, 4096, K): 64 full tiles, which the ring-buffered kernel takes as 128 tiles of 128 x 256;
# (2048, 12288, K): 384 full tiles = one round of 256 and a last round of 128, whose columns are computed on
# 128 x 256 tiles by a second launch
GEMM_SHAPES = [(300, 200, 136), (512, 384, 256), (130, 72, 8), (4096, 4096, 128), (4072, 4088, 200), (4096, 4096, 64),
               (4096, 4096, 192), (1024, 4096, 192), (1024, 4096, 64), (2048, 12288, 128)]


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("shape", GEMM_SHAPES)
def test_gemm_forward_layout_bias(ctx, orc, shape, bf16):
    """C = x[M,K] . W[K,N] + b: A row-major in k, B stored k-major (the forward projections)."""
    M, N, K = shape
    if not bf16 and M * N * K > 1e9:
        pytest.skip("fp32 ALU path is for the small configuration")
    x, xv = dev_act(_rand(1, (M, K)), bf16)
    w, wv = dev_act(_rand(2, (K, N), 0.05), bf16)
    b = _rand(3, (N,))
    bd = dev_f32(b)
    out = empty_act((M, N), bf16)
    ctx.gemm(dtype=DT[bf16], a_kmajor=0, b_kmajor=1, M=M, N=N, K=K, lda=K, ldb=N, ldc=N, epilogue=pwb.PW_EPI_BIAS,
             out_dtype=DT[bf16], accumulate=0, A=ptr(x), B=ptr(w), bias=ptr(bd), C=ptr(out))
    ctx.synchronize()
    ref = orc.linear_fwd(xv, wv, b.astype(np.float64))
    assert_close(host(out), ref, 4e-3 if bf16 else 2e-6)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("shape", GEMM_SHAPES[:3] + [(4096, 4096, 128), (4096, 4096, 64), (4096, 4096, 192), (1024, 4096, 192),
                                                    (2048, 12288, 64)])
def test_gemm_dgrad_and_wgrad_layouts(ctx, orc, shape, bf16):
    """dx = dy . W^T (B stored [n][k]) and dW = x^T . dy (both operands k-major), fp32 accumulate-into."""
    M, N, K = shape          # M tokens, N = in features, K = out features
    if not bf16 and M * N * K > 1e9:
        pytest.skip("fp32 ALU path is for the small configuration")
    if bf16 and (N % 8 or K % 8 or M % 8):
        pytest.skip("bf16 operands need 16-byte aligned rows")
    dy, dyv = dev_act(_rand(4, (M, K)), bf16)
    w, wv = dev_act(_rand(5, (N, K), 0.05), bf16)
    x, xv = dev_act(_rand(6, (M, N)), bf16)
    dx = empty_act((M, N), bf16)
    ctx.gemm(dtype=DT[bf16], a_kmajor=0, b_kmajor=0, M=M, N=N, K=K, lda=K, ldb=K, ldc=N, epilogue=pwb.PW_EPI_STORE,
             out_dtype=DT[bf16], accumulate=0, A=ptr(dy), B=ptr(w), C=ptr(dx))
    base = _rand(7, (N, K))
    dw = dev_f32(base)
    for acc in (1, 0):
        ctx.gemm(dtype=DT[bf16], a_kmajor=1, b_kmajor=1, M=N, N=K, K=M, lda=N, ldb=K, ldc=K,
                 epilogue=pwb.PW_EPI_STORE, out_dtype=pwb.PW_F32, accumulate=acc, A=ptr(x), B=ptr(dy), C=ptr(dw))
        ctx.synchronize()
        rdx, rdw, _ = orc.linear_bwd(xv, wv, dyv)
        want = rdw + base if acc else rdw
        assert_close(host(dw), want, 2e-6, acc)
    assert_close(host(dx), rdx, 4e-3 if bf16 else 2e-6)


# ragged (register-staged kernel), 64 full tiles (ring kernel on 128 x 256 tiles), 256 full tiles (ring kernel)
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("shape", [(264, 328, 192), (1024, 4096, 128), (4096, 4096, 128), (2048, 12288, 64)])
def test_gemm_fused_epilogues(ctx, orc, bf16, shape):
    M, N, K = shape
    if not bf16 and M * N * K > 1e8:
        pytest.skip("fp32 ALU path is for the small configuration")
    x, xv = dev_act(_rand(8, (M, K)), bf16)
    w, wv = dev_act(_rand(9, (K, N), 0.08), bf16)
    b = _rand(10, (N,), 0.5)
    bd = dev_f32(b)
    lin = orc.linear_fwd(xv, wv, b.astype(np.float64))
    common = dict(dtype=DT[bf16], a_kmajor=0, b_kmajor=1, M=M, N=N, K=K, lda=K, ldb=N, ldc=N, accumulate=0,
                  A=ptr(x), B=ptr(w))
    # bias + GELU, both the pre-activation and the activation are kept
    u, h = empty_act((M, N), bf16), empty_act((M, N), bf16)
    ctx.gemm(epilogue=pwb.PW_EPI_BIAS_GELU, out_dtype=DT[bf16], bias=ptr(bd), C=ptr(u), C2=ptr(h), **common)
    # bias + residual into the fp32 stream
    res = _rand(11, (M, N))
    resd, xo = dev_f32(res), torch.empty((M, N), dtype=torch.float32, device="cuda")
    ctx.gemm(epilogue=pwb.PW_EPI_BIAS_RESIDUAL, out_dtype=pwb.PW_F32, bias=ptr(bd), aux=ptr(resd), C=ptr(xo), **common)
    # product times gelu'(aux)
    pre, prev = dev_act(_rand(12, (M, N), 1.5), bf16)
    du = empty_act((M, N), bf16)
    ctx.gemm(epilogue=pwb.PW_EPI_GELU_BWD, out_dtype=DT[bf16], aux=ptr(pre), C=ptr(du), **common)
    ctx.synchronize()
    tol = 4e-3 if bf16 else 2e-6
    assert_close(host(u), lin, tol)
    assert_close(host(h), orc.gelu_fwd(lin), tol * 1.5)
    assert_close(host(xo), lin + res, 2e-6 if not bf16 else 1e-5)
    nobias = orc.linear_fwd(xv, wv)
    assert_close(host(du), orc.gelu_bwd(prev, nobias), tol)


@pytest.mark.parametrize("bf16", [False, True])
def test_gemm_pair_small_problems_and_rejection(ctx, orc, bf16):
    """Two problems that do not qualify for a shared launch still give both results; one bad argument set
    means neither runs."""
    (M0, N0, K0), (M1, N1, K1) = (136, 72, 64), (40, 264, 200)
    x0, x0v = dev_act(_rand(20, (M0, K0)), bf16)
    w0, w0v = dev_act(_rand(21, (K0, N0), 0.1), bf16)
    x1, x1v = dev_act(_rand(22, (M1, K1)), bf16)
    w1, w1v = dev_act(_rand(23, (K1, N1), 0.1), bf16)
    c0 = torch.full((M0, N0), 7.0, device="cuda")
    c1 = torch.full((M1, N1), 7.0, device="cuda")
    def args(x, w, c, M, N, K):
        return dict(dtype=DT[bf16], a_kmajor=0, b_kmajor=1, M=M, N=N, K=K, lda=K, ldb=N, ldc=N,
                    epilogue=pwb.PW_EPI_STORE, out_dtype=pwb.PW_F32, accumulate=0, A=ptr(x), B=ptr(w), C=ptr(c))
    with pytest.raises(pwb.PwError):
        ctx.gemm_pair(args(x0, w0, c0, M0, N0, K0), {**args(x1, w1, c1, M1, N1, K1), "ldb": 8})
    ctx.synchronize()
    assert (host(c0) == 7.0).all() and (host(c1) == 7.0).all()
    ctx.gemm_pair(args(x0, w0, c0, M0, N0, K0), args(x1, w1, c1, M1, N1, K1))
    ctx.synchronize()
    assert_close(host(c0), orc.linear_fwd(x0v, w0v), 2e-6)
    assert_close(host(c1), orc.linear_fwd(x1v, w1v), 2e-6)


# ---- fused epilogues of the step's two largest non-GEMM passes -------------------------------------------

def _adam_case(seed, n_in, n_out, ntok):
    x, xv = dev_act(_rand(seed, (ntok, n_in)), True)
    dy, dyv = dev_act(_rand(seed + 1, (ntok, n_out), 0.3), True)
    w = _rand(seed + 2, (n_in, n_out), 0.02).astype(np.float32)
    m = _rand(seed + 3, (n_in, n_out), 0.05).astype(np.float32)
    # second moments bounded away from zero: where v and g are both tiny the update is a quotient of two roundings
    v = ((0.05 + np.abs(_rand(seed + 4, (n_in, n_out), 0.05))) ** 2).astype(np.float32)
    return dict(x=x, xv=xv, dy=dy, dyv=dyv, w=w, m=m, v=v, wd=dev_f32(w), md=dev_f32(m), vd=dev_f32(v),
                wlp=torch.zeros((n_in, n_out), dtype=torch.bfloat16, device="cuda"),
                g=torch.full((n_in, n_out), float("nan"), device="cuda"), n_in=n_in, n_out=n_out, ntok=ntok)


def _adam_gemm_kw(c, hp, t, store_g):
    ep = pwb.AdamEpilogue(ptr(c["wd"]), ptr(c["md"]), ptr(c["vd"]), ptr(c["wlp"]), *hp, t)
    return dict(dtype=pwb.PW_BF16, a_kmajor=1, b_kmajor=1, M=c["n_in"], N=c["n_out"], K=c["ntok"], lda=c["n_in"],
                ldb=c["n_out"], ldc=c["n_out"], epilogue=pwb.PW_EPI_ADAM, out_dtype=pwb.PW_F32, accumulate=0,
                A=ptr(c["x"]), B=ptr(c["dy"]), C=ptr(c["g"]) if store_g else None, adam=ep)


def _check_adam_case(orc, c, hp, t, store_g):
    _, g, _ = orc.linear_bwd(c["xv"], np.zeros((c["n_in"], c["n_out"])), c["dyv"])
    rw, rm, rv = orc.adam(c["w"], c["m"], c["v"], g, *[np.float32(h) for h in hp], t)
    if store_g:
        assert_close(host(c["g"]), g, 2e-6, "g")
    assert_close(host(c["md"]), rm, 1e-5, "m")
    assert_close(host(c["vd"]), rv, 1e-5, "v")
    w64 = c["w"].astype(np.float64)
    # the update is small against w: compare it, and allow the fp32 storage of w on top
    assert_close(host(c["wd"]) - w64, rw - w64, 1e-4, "dw", norm_slack=1e-3, extra=np.abs(w64) * 1.2e-7)
    assert np.array_equal(c["wlp"].float().cpu().numpy(), I.round_to_bf16(c["wd"].cpu().numpy()))   # bf16 copy = RNE(w)


@pytest.mark.parametrize("t", [1, 3])
def test_gemm_with_adam_epilogue(ctx, orc, t):
    """dW = x^T . dy with the Adam update of W in the GEMM's epilogue (26 bytes of optimizer traffic per parameter,
    the gradient stored only on request): against the oracle's linear backward followed by the oracle's Adam."""
    hp = (1e-3, 0.9, 0.95, 1e-8)
    c = _adam_case(80, 2048, 5120, 192)                   # 160 tiles of 256 x 256: one launch of the ring kernel
    if t == 1:
        c["md"].zero_(), c["vd"].zero_()
        c["m"][:], c["v"][:] = 0, 0
    ctx.gemm(**_adam_gemm_kw(c, hp, t, store_g=True))
    ctx.synchronize()
    _check_adam_case(orc, c, hp, t, store_g=True)
    # without the gradient output, from the same state: same update
    c2 = _adam_case(80, 2048, 5120, 192)
    if t == 1:
        c2["md"].zero_(), c2["vd"].zero_()
        c2["m"][:], c2["v"][:] = 0, 0
    ctx.gemm(**_adam_gemm_kw(c2, hp, t, store_g=False))
    ctx.synchronize()
    for k in ("wd", "md", "vd", "wlp"):
        assert torch.equal(c[k], c2[k]), k
    assert torch.isnan(c2["g"]).all()


def test_gemm_group_with_adam_epilogues_and_bias_gradient(ctx, orc):
    """Two weight gradients sharing one launch (128 + 32 tiles), both with the Adam epilogue, one with the bias
    gradient riding along - the QKV / out-projection pair of a layer."""
    hp = (1e-3, 0.9, 0.95, 1e-8)
    a, b = _adam_case(90, 2048, 4096, 128), _adam_case(95, 2048, 1024, 128)
    dbias = torch.full((4096,), float("nan"), device="cuda")
    ctx.gemm_group([{**_adam_gemm_kw(a, hp, 2, True), "b_colsum": ptr(dbias)}, _adam_gemm_kw(b, hp, 2, False)])
    ctx.synchronize()
    _check_adam_case(orc, a, hp, 2, True)
    _check_adam_case(orc, b, hp, 2, False)
    assert_close(host(dbias), a["dyv"].sum(axis=0), 1e-5)
    # what the kernel cannot take is refused before anything runs: ragged shape, row-major operand, accumulate
    w0 = a["wd"].clone()
    for bad in (dict(M=2040, lda=2040), dict(a_kmajor=0), dict(accumulate=1)):
        with pytest.raises(pwb.PwError):
            ctx.gemm(**{**_adam_gemm_kw(a, hp, 2, True), **bad})
    ctx.synchronize()
    assert torch.equal(w0, a["wd"])


def test_profile_reports_the_launches_by_shape(ctx):
    """The measurement aid's per-shape table: three launches of one shape and one of another, bracketed by events."""
    x = torch.zeros(512 * 512, dtype=torch.bfloat16, device="cuda")
    c = torch.empty(512 * 512, dtype=torch.bfloat16, device="cuda")

    def run(K):
        ctx.gemm(dtype=pwb.PW_BF16, a_kmajor=0, b_kmajor=1, M=512, N=512, K=K, lda=K, ldb=512, ldc=512, accumulate=0,
                 epilogue=pwb.PW_EPI_STORE, out_dtype=pwb.PW_BF16, A=ptr(x), B=ptr(x), C=ptr(c))
    ctx.profile_begin()
    for K in (256, 512, 512, 512):
        run(K)
    n, ms, fl = ctx.profile_end()
    rows = ctx.profile_gemm_shapes()
    assert n == 4 and ms > 0 and fl == 2.0 * 512 * 512 * (256 + 3 * 512)
    assert sorted((r["K"], r["launches"]) for r in rows) == [(256, 1), (512, 3)]
    assert all(r["M"] == 512 and r["N"] == 512 and r["members"] == 1 and r["a_kmajor"] == 0 and r["b_kmajor"] == 1
               and r["epilogue"] == pwb.PW_EPI_STORE for r in rows)
    assert abs(sum(r["total_ms"] for r in rows) - ms) < 1e-6 * max(ms, 1.0) + 1e-9
    assert sum(r["total_flops"] for r in rows) == fl


def test_lm_head_fused_with_the_loss(ctx, orc):
    """The LM-head GEMM with the loss in its epilogue: a first pass over y . Wh leaves only softmax statistics per
    64-column group and the targets' logits, a second pass writes (softmax - onehot) / N in bf16 - the logits
    themselves are never stored.  Against the oracle's linear forward + softmax cross-entropy."""
    B, T, d, V = 4, 512, 256, 8192                        # 8 x 32 tiles
    N = B * T
    y, yv = dev_act(_rand(100, (N, d)), True)
    wh, whv = dev_act(_rand(101, (d, V), 0.08), True)
    tok = I.tokens(102, 1, (B, T + 1), V)
    tok[1, 5], tok[2, 7] = -3, V + 11                      # out-of-range ids are clamped, as everywhere
    tokd = dev_i32(tok)
    part = torch.full((N, V // 64, 2), float("nan"), device="cuda")
    zt, lse, rows, loss = (torch.full((n,), float("nan"), device="cuda") for n in (N, N, N, 1))
    dz = torch.full((N, V), float("nan"), dtype=torch.bfloat16, device="cuda")
    common = dict(dtype=pwb.PW_BF16, a_kmajor=0, b_kmajor=1, M=N, N=V, K=d, lda=d, ldb=V, ldc=V, accumulate=0,
                  A=ptr(y), B=ptr(wh))
    xe = pwb.XentEpilogue(ptr(tokd), T, ptr(part), ptr(zt), ptr(lse), 1.0 / N)
    ctx.gemm(epilogue=pwb.PW_EPI_XENT_STATS, out_dtype=pwb.PW_BF16, C=None, xent=xe, **common)
    ctx.op("xent_from_stats", ptr(part), ptr(zt), ptr(lse), ptr(rows), ptr(loss), N, V // 64)
    ctx.gemm(epilogue=pwb.PW_EPI_XENT_GRAD, out_dtype=pwb.PW_BF16, C=ptr(dz), xent=xe, **common)
    ctx.synchronize()
    z = orc.linear_fwd(yv, whv)
    tgt = np.clip(tok[:, 1:].reshape(-1), 0, V - 1)
    rl, rdz = orc.softmax_xent(z, tgt)
    zmax = z.max(axis=1)
    rlse = np.log(np.exp(z - zmax[:, None]).sum(axis=1)) + zmax
    assert abs(host(loss)[0] - rl) / rl < 1e-5
    assert_close(host(lse), rlse, 1e-5, "lse")
    assert_close(host(zt), z[np.arange(N), tgt], 1e-5, "target logits")
    assert_close(host(rows), rlse - z[np.arange(N), tgt], 1e-5, "row losses")
    assert_close(host(dz), rdz, 6e-3, "dz")
    with pytest.raises(pwb.PwError):                       # ragged vocabulary: refused, nothing runs
        ctx.gemm(epilogue=pwb.PW_EPI_XENT_STATS, out_dtype=pwb.PW_BF16, C=None, xent=xe, **{**common, "N": V - 8})


def test_gemm_rejects_what_the_kernel_cannot_take(ctx):
    a = torch.zeros(64 * 64, dtype=torch.bfloat16, device="cuda")
    c = torch.zeros(64 * 64, dtype=torch.float32, device="cuda")
    base = dict(dtype=pwb.PW_BF16, a_kmajor=0, b_kmajor=0, M=16, N=16, K=20, lda=20, ldb=20, ldc=16,
                epilogue=pwb.PW_EPI_STORE, out_dtype=pwb.PW_F32, accumulate=0, A=ptr(a), B=ptr(a), C=ptr(c))
    with pytest.raises(pwb.PwError):
        ctx.gemm(**base)                                   # K not a multiple of 8
    with pytest.raises(pwb.PwError):
        ctx.gemm(**{**base, "K": 16, "lda": 8, "ldb": 16})  # lda < K
    with pytest.raises(pwb.PwError):
        ctx.gemm(**{**base, "K": 16, "lda": 16, "ldb": 16, "A": ptr(a) + 2})   # misaligned
    with pytest.raises(pwb.PwError):
        ctx.gemm(**{**base, "K": 16, "lda": 16, "ldb": 16, "epilogue": pwb.PW_EPI_BIAS_RESIDUAL})   # no aux
    ctx.gemm(**{**base, "K": 16, "lda": 16, "ldb": 16, "M": 0})    # empty problem: accepted, nothing launched
    ctx.synchronize()


# ---- LayerNorm ----------------------------------------------------------------------------------------

@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("N,d", [(37, 256), (5, 1000), (600, 2048), (3, 8192), (2100, 2048), (1030, 512), (70, 4096)])
def test_layernorm_forward_backward(ctx, orc, N, d, bf16):
    x = _rand(20, (N, d), 2.0) + 0.5
    g, b = 1 + _rand(21, (d,), 0.1), _rand(22, (d,), 0.1)
    xd, gd, bd = dev_f32(x), dev_f32(g), dev_f32(b)
    y = empty_act((N, d), bf16)
    mean, rstd = torch.empty(N, device="cuda"), torch.empty(N, device="cuda")
    ctx.op("layernorm_fwd", DT[bf16], ptr(xd), ptr(gd), ptr(bd), ptr(y), ptr(mean), ptr(rstd), N, d)
    ry, rmean, rrstd = orc.layernorm_fwd(x, g, b)
    dy, dyv = dev_act(_rand(23, (N, d)), bf16)
    dres = _rand(24, (N, d))
    dresd = dev_f32(dres)
    dx = torch.empty((N, d), device="cuda")
    dxlp = empty_act((N, d), bf16) if bf16 else None
    dg, db, dsum = dev_f32(np.ones(d)), dev_f32(np.ones(d)), dev_f32(np.ones(d))
    ws = torch.empty(pwb.lib().pw_layernorm_bwd_ws_floats(N, d), device="cuda")
    ctx.op("layernorm_bwd", DT[bf16], ptr(dy), ptr(xd), ptr(gd), ptr(mean), ptr(rstd), ptr(dresd), ptr(dx), ptr(dxlp),
           ptr(dg), ptr(db), ptr(dsum), ptr(ws), N, d, 1)
    # without the residual input and the optional outputs, overwrite mode
    dx0, dg0, db0 = torch.empty((N, d), device="cuda"), dev_f32(np.ones(d)), dev_f32(np.ones(d))
    ctx.op("layernorm_bwd", DT[bf16], ptr(dy), ptr(xd), ptr(gd), ptr(mean), ptr(rstd), None, ptr(dx0), None,
           ptr(dg0), ptr(db0), None, ptr(ws), N, d, 0)
    ctx.synchronize()
    assert_close(host(y), ry, 4e-3 if bf16 else 2e-6)
    assert_close(host(mean), rmean, 1e-5)
    assert_close(host(rstd), rrstd, 1e-5)
    rdx, rdg, rdb = orc.layernorm_bwd(dyv, x, g)
    assert_close(host(dx), rdx + dres, 1e-5)
    assert_close(host(dg), rdg + 1.0, 1e-5)                                            # accumulate = 1 adds
    assert_close(host(db), rdb + 1.0, 1e-5)
    assert_close(host(dsum), (rdx + dres).sum(axis=0) + 1.0, 1e-5)                     # column sums of dx
    assert_close(host(dx0), rdx, 1e-5)
    assert_close(host(dg0), rdg, 1e-5)
    assert_close(host(db0), rdb, 1e-5)
    if bf16:
        assert_close(host(dxlp), rdx + dres, 4e-3)


# ---- attention ----------------------------------------------------------------------------------------

@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("B,T,H,hd", [(2, 200, 2, 64), (1, 130, 3, 128), (2, 1, 1, 64), (1, 384, 2, 128)])
def test_attention_forward_backward(ctx, orc, B, T, H, hd, bf16):
    d = H * hd
    qkv, qkvv = dev_act(_rand(30, (B * T, 3 * d), 1.0), bf16)
    o = empty_act((B * T, d), bf16)
    lse = torch.empty((B, H, T), device="cuda")
    ctx.op("attention_fwd", DT[bf16], ptr(qkv), ptr(o), ptr(lse), B, T, H, hd)
    ctx.synchronize()
    ro = orc.attention_fwd(qkvv, B, T, H, hd)
    assert_close(host(o), ro, 6e-3 if bf16 else 1e-5)
    # log-sum-exp of the scaled causal scores, brute force for a few rows
    r = qkvv.reshape(B, T, 3, H, hd)
    for (b, h, i) in [(0, 0, 0), (B - 1, H - 1, T - 1), (0, H - 1, T // 2)]:
        s = r[b, : i + 1, 1, h] @ r[b, i, 0, h] / np.sqrt(hd)
        want = np.log(np.exp(s - s.max()).sum()) + s.max()
        assert abs(host(lse)[b, h, i] - want) < (2e-2 if bf16 else 1e-4)
    dout, doutv = dev_act(_rand(31, (B * T, d)), bf16)
    dqkv = empty_act((B * T, 3 * d), bf16)
    delta = torch.empty((B, H, T), device="cuda")
    ctx.op("attention_bwd", DT[bf16], ptr(qkv), ptr(o), ptr(dout), ptr(lse), ptr(delta), ptr(dqkv), B, T, H, hd)
    ctx.synchronize()
    rd = orc.attention_bwd(qkvv, doutv, B, T, H, hd)
    got = host(dqkv)
    for name, sl in (("dq", slice(0, d)), ("dk", slice(d, 2 * d)), ("dv", slice(2 * d, 3 * d))):
        assert_close(got[:, sl], rd[:, sl], 1.5e-2 if bf16 else 1e-5, name)


def _mha_case(ctx, orc, bf16, B, Tq, Tk, H, hd, causal, packed_kv):
    """General attention against the oracle: q from its own array, k and v either packed [K|V] rows or separate."""
    d = H * hd
    es = 2 if bf16 else 4
    q, qv = dev_act(_rand(32, (B * Tq, d), 1.0), bf16)
    if packed_kv:
        kv, kvv = dev_act(_rand(33, (B * Tk, 2 * d), 1.0), bf16)
        kp, vp, ldkv, kh, vh = ptr(kv), ptr(kv) + d * es, 2 * d, kvv[:, :d], kvv[:, d:]
    else:
        k, kh = dev_act(_rand(33, (B * Tk, d), 1.0), bf16)
        v, vh = dev_act(_rand(34, (B * Tk, d), 1.0), bf16)
        kp, vp, ldkv = ptr(k), ptr(v), d
    a = pwb.MhaArgs(DT[bf16], ptr(q), kp, vp, d, ldkv, B, Tq, Tk, H, hd, int(causal))
    o, o_lo = empty_act((B * Tq, d), bf16), empty_act((B * Tq, d), bf16)
    lse = torch.empty((B, H, Tq), device="cuda")
    ctx.mha_fwd(a, ptr(o), ptr(lse), o_lo=ptr(o_lo))
    ctx.synchronize()
    ro = orc.mha_fwd(qv, kh, vh, B, Tq, Tk, H, hd, causal=causal)
    # o_lo holds what rounding O left over (nothing in fp32); the sum is the kernel's fp32 result, itself exact only
    # as far as the bf16 probabilities of the second product allow
    assert_close(host(o) + host(o_lo), ro, 4e-3 if bf16 else 1e-5)
    assert np.abs(host(o_lo)).max() <= (np.abs(host(o)).max() * 2.0 ** -8 if bf16 else 0.0)
    assert_close(host(o), ro, 6e-3 if bf16 else 1e-5)
    qr, kr = qv.reshape(B, Tq, H, hd), np.ascontiguousarray(kh).reshape(B, Tk, H, hd)
    for (b, h, i) in [(0, 0, 0), (B - 1, H - 1, Tq - 1), (0, H - 1, Tq // 2)]:
        s = kr[b, : (i + 1 if causal else Tk), h] @ qr[b, i, h] / np.sqrt(hd)
        want = np.log(np.exp(s - s.max()).sum()) + s.max()
        assert abs(host(lse)[b, h, i] - want) < (2e-2 if bf16 else 1e-4)
    dout, doutv = dev_act(_rand(35, (B * Tq, d)), bf16)
    dq = empty_act((B * Tq, d), bf16)
    dkv = empty_act((B * Tk, 2 * d), bf16)             # gradients always packed [dK|dV] here
    delta = torch.empty((B, H, Tq), device="cuda")
    ctx.mha_bwd(a, ptr(o), ptr(dout), ptr(lse), ptr(delta), ptr(dq), d, ptr(dkv), ptr(dkv) + d * es, 2 * d, o_lo=ptr(o_lo))
    ctx.synchronize()
    rdq, rdk, rdv = orc.mha_bwd(qv, kh, vh, doutv, B, Tq, Tk, H, hd, causal=causal)
    tol = 1.5e-2 if bf16 else 1e-5
    assert_close(host(dq), rdq, tol)
    assert_close(host(dkv)[:, :d], rdk, tol)
    assert_close(host(dkv)[:, d:], rdv, tol)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("B,Tq,Tk,H,hd", [(2, 70, 200, 2, 64), (1, 130, 97, 3, 128), (2, 5, 1, 1, 64), (1, 300, 384, 2, 128),
                                          (2, 129, 64, 2, 128)])
def test_unmasked_attention_with_separate_lengths(ctx, orc, B, Tq, Tk, H, hd, bf16):
    _mha_case(ctx, orc, bf16, B, Tq, Tk, H, hd, causal=False, packed_kv=True)


def test_causal_attention_block_order_with_partial_problem_groups(ctx, orc):
    """Under the causal mask the workgroups of several problems are interleaved, longest blocks first, in groups
    sized from the number of 128-row blocks per problem: 9 problems of 5 blocks give one group of 9 in the forward
    and dQ kernels and groups of 7 and 2 in the dK/dV kernel, with a ragged last block."""
    _mha_case(ctx, orc, True, 3, 520, 520, 3, 128, causal=True, packed_kv=False)


@pytest.mark.parametrize("bf16", [False, True])
def test_general_attention_entry_point_other_layouts(ctx, orc, bf16):
    _mha_case(ctx, orc, bf16, 2, 150, 150, 2, 128, causal=True, packed_kv=False)    # causal, k and v separate
    _mha_case(ctx, orc, bf16, 1, 96, 96, 2, 64, causal=False, packed_kv=False)      # encoder self-attention shape


def test_attention_output_remainder_keeps_query_gradient_accurate(ctx, orc):
    """Near-uniform attention over keys and values that share a large common component (what an encoder's output
    looks like at initialisation): delta = rowsum(dO * O) from the bf16-rounded O alone puts several per cent of
    error into dq and dk; with the rounding remainder kept by the forward call they meet the bf16 bar."""
    B, Tq, Tk, H, hd = 1, 256, 1024, 2, 128
    d = H * hd
    common = _rand(50, (1, 2 * d), 2.0)
    q, qv = dev_act(_rand(51, (B * Tq, d), 0.05), True)
    kv, kvv = dev_act(_rand(52, (B * Tk, 2 * d), 1.0) + common, True)
    dout, doutv = dev_act(_rand(53, (B * Tq, d)), True)
    a = pwb.MhaArgs(pwb.PW_BF16, ptr(q), ptr(kv), ptr(kv) + d * 2, d, 2 * d, B, Tq, Tk, H, hd, 0)
    rdq, rdk, rdv = orc.mha_bwd(qv, kvv[:, :d], kvv[:, d:], doutv, B, Tq, Tk, H, hd)
    errs = {}
    for keep in (False, True):
        o, o_lo = empty_act((B * Tq, d), True), empty_act((B * Tq, d), True)
        lse, delta = torch.empty((B, H, Tq), device="cuda"), torch.empty((B, H, Tq), device="cuda")
        dq, dkv = empty_act((B * Tq, d), True), empty_act((B * Tk, 2 * d), True)
        lo = ptr(o_lo) if keep else 0
        ctx.mha_fwd(a, ptr(o), ptr(lse), o_lo=lo)
        ctx.mha_bwd(a, ptr(o), ptr(dout), ptr(lse), ptr(delta), ptr(dq), d, ptr(dkv), ptr(dkv) + d * 2, 2 * d, o_lo=lo)
        ctx.synchronize()
        errs[keep] = (rel_l2(host(dq), rdq), rel_l2(host(dkv)[:, :d], rdk), rel_l2(host(dkv)[:, d:], rdv))
        if keep:   # with 1024 keys of similar weight the bf16 probabilities average out: o + o_lo is O to many more bits
            ro = orc.mha_fwd(qv, kvv[:, :d], kvv[:, d:], B, Tq, Tk, H, hd)
            assert rel_l2(host(o) + host(o_lo), ro) < 0.2 * rel_l2(host(o), ro)
    print("dq, dk, dv errors without / with the remainder:", errs[False], errs[True])
    assert max(errs[True]) < 1.5e-2
    for got, want, name in ((host(dq), rdq, "dq"), (host(dkv)[:, :d], rdk, "dk"), (host(dkv)[:, d:], rdv, "dv")):
        assert_close(got, want, 1.5e-2, name)          # the last pass of the loop kept the remainder
    assert errs[False][0] > 3 * errs[True][0]          # what the remainder is for


def test_general_attention_rejects_bad_arguments(ctx):
    q = torch.zeros((64, 128), device="cuda")
    lse = torch.zeros((1, 1, 64), device="cuda")
    ok = dict(dtype=pwb.PW_F32, q=ptr(q), k=ptr(q), v=ptr(q), ldq=128, ldkv=128, B=1, Tq=64, Tk=64, H=1, hd=128, causal=0)
    for bad in (dict(hd=96), dict(Tk=0), dict(ldkv=64), dict(causal=1, Tk=32), dict(k=0), dict(dtype=7)):
        a = pwb.MhaArgs(**{**ok, **bad})
        with pytest.raises(pwb.PwError):
            ctx.mha_fwd(a, ptr(q), ptr(lse))
    ctx.mha_fwd(pwb.MhaArgs(**ok), ptr(q), ptr(lse))
    ctx.synchronize()


# ---- softmax cross-entropy ----------------------------------------------------------------------------

@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("B,T,V", [(3, 5, 1024), (2, 7, 4096), (1, 3, 32768), (2, 2, 8)])
def test_softmax_xent(ctx, orc, B, T, V, bf16):
    N = B * T
    z, zv = dev_act(_rand(40, (N, V), 2.0), bf16)
    tok = I.tokens(41, 1, (B, T + 1), V)
    tokd = dev_i32(tok)
    loss, rows = torch.empty(1, device="cuda"), torch.empty(N, device="cuda")
    ctx.op("softmax_xent", DT[bf16], ptr(z), ptr(tokd), ptr(loss), ptr(rows), B, T, V)
    ctx.synchronize()
    rl, rdz = orc.softmax_xent(zv, tok[:, 1:].reshape(-1))
    assert abs(host(loss)[0] - rl) / rl < 1e-5
    assert_close(host(z), rdz, 6e-3 if bf16 else 1e-5)
    if not bf16:
        assert np.abs(host(z).sum(axis=1)).max() < 1e-6     # rows of dlogits sum to 0


# ---- embedding ----------------------------------------------------------------------------------------

def test_embedding_forward_is_bit_exact_and_backward_is_deterministic(ctx, orc):
    B, T, d, V = 4, 129, 256, 97          # V small: many repeated ids
    tok = I.tokens(50, 1, (B, T + 1), V)
    tok[0, :40] = 5                        # one id repeated many times, in a row and across rows
    tok[1, 10:30] = 5
    wte, wpe = _rand(51, (V, d), 0.02), _rand(52, (T, d), 0.02)
    tokd, wted, wped = dev_i32(tok), dev_f32(wte), dev_f32(wpe)
    x = torch.empty((B * T, d), device="cuda")
    ctx.op("embedding_fwd", ptr(tokd), ptr(wted), ptr(wped), ptr(x), B, T, d, V)
    ctx.synchronize()
    inp = tok[:, :T]
    want = (wte[inp.reshape(-1)] + np.tile(wpe, (B, 1))).astype(np.float32)      # one fp32 add per element
    assert np.array_equal(x.cpu().numpy(), want)
    # the oracle adds in double, where the sum of two fp32 values is exact; rounded once it must give the same bits
    assert np.array_equal(x.cpu().numpy(), orc.embedding_fwd(inp, wte, wpe).astype(np.float32))
    dx = _rand(53, (B * T, d))
    dxd = dev_f32(dx)
    outs = []
    for _ in range(2):
        dwte = torch.full((V, d), 7.0, device="cuda")        # stale contents must be overwritten
        dwpe = torch.full((T, d), 7.0, device="cuda")
        ctx.op("embedding_bwd", ptr(tokd), ptr(dxd), ptr(dwte), ptr(dwpe), B, T, d, V)
        ctx.synchronize()
        outs.append((dwte.cpu().numpy(), dwpe.cpu().numpy()))
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])
    rwte, rwpe = orc.embedding_bwd(inp, dx, V)
    assert_close(outs[0][0], rwte, 1e-6)
    assert_close(outs[0][1], rwpe, 1e-6)
    unused = sorted(set(range(V)) - set(inp.reshape(-1).tolist()))
    for u in unused:
        assert (outs[0][0][u] == 0).all()


def test_embedding_backward_handles_one_id_everywhere(ctx, orc):
    """Degenerate case: every position holds the same id (the list of matches exceeds one LDS batch)."""
    B, T, d, V = 3, 1000, 64, 11
    tok = np.full((B, T + 1), 4, dtype=np.int32)
    dx = _rand(54, (B * T, d))
    tokd, dxd = dev_i32(tok), dev_f32(dx)
    dwte, dwpe = torch.empty((V, d), device="cuda"), torch.empty((T, d), device="cuda")
    ctx.op("embedding_bwd", ptr(tokd), ptr(dxd), ptr(dwte), ptr(dwpe), B, T, d, V)
    ctx.synchronize()
    rwte, _ = orc.embedding_bwd(tok[:, :T], dx, V)
    assert_close(host(dwte), rwte, 1e-5)


# ---- column sums and optimisers -----------------------------------------------------------------------

@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("rows,cols", [(513, 768), (8, 64), (2048, 8192), (1, 12)])
def test_colsum(ctx, rows, cols, bf16):
    a, av = dev_act(_rand(60, (rows, cols)), bf16)
    out = dev_f32(np.full(cols, 3.0))
    ws = torch.empty(pwb.lib().pw_colsum_ws_floats(rows, cols), device="cuda")
    ctx.op("colsum", DT[bf16], ptr(a), ptr(out), ptr(ws), rows, cols, 1)
    ctx.synchronize()
    assert_close(host(out), av.sum(axis=0) + 3.0, 1e-5)
    ctx.op("colsum", DT[bf16], ptr(a), ptr(out), ptr(ws), rows, cols, 0)
    ctx.synchronize()
    assert_close(host(out), av.sum(axis=0), 1e-5)


@pytest.mark.parametrize("n", [1, 1023, 1 << 20])
def test_sgd_and_adam_kernels(ctx, orc, n):
    w, g = _rand(70, (n,)), _rand(71, (n,), 0.1)
    g[: n // 3] = 0.0
    wd, gd = dev_f32(w), dev_f32(g)
    ctx.op("sgd", ptr(wd), ptr(gd), n, 0.01)
    ctx.synchronize()
    assert_close(host(wd), orc.sgd(w.astype(np.float64), g.astype(np.float64), np.float32(0.01)), 1e-7)
    wd, md, vd = dev_f32(w), dev_f32(np.zeros(n)), dev_f32(np.zeros(n))
    wlp = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    rw, rm, rv = w.astype(np.float64), np.zeros(n), np.zeros(n)
    lr, b1, b2, eps = 1e-3, 0.9, 0.95, 1e-8
    for t in (1, 2, 3):
        ctx.op("adam", ptr(wd), ptr(md), ptr(vd), ptr(gd), ptr(wlp), n, lr, b1, b2, eps, t)
        rw, rm, rv = orc.adam(rw, rm, rv, g.astype(np.float64), np.float32(lr), np.float32(b1), np.float32(b2),
                              np.float32(eps), t)
    ctx.synchronize()
    assert np.abs(host(wd) - rw).max() < 1e-6            # identical gradient: the kernel itself is held to 1e-6
    assert_close(host(md), rm, 1e-6)
    assert_close(host(vd), rv, 1e-6)
    assert np.array_equal(wlp.float().cpu().numpy(), I.round_to_bf16(wd.cpu().numpy()))   # bf16 copy is RNE of w
