"""The entry point that allocates nothing (pw_op_layernorm_bwd_noalloc): through the C boundary against the
existing entry point with a caller workspace - same kernels, so the same bits - and against the oracle, on two calls
in a row of which the second is smaller (the fixed array still holds the first call's block sums), then on a
ragged third; sizes beyond the fixed array are refused with nothing written."""
import numpy as np
import pytest
import torch

from paper_2203_12533_amd import binding as pwb
from paper_2203_12533_amd import inputs as I
from gpu_util import DT, assert_close, dev_act, dev_f32, empty_act, host, ptr

pytestmark = pytest.mark.gpu


def _rand(seed, shape, std=1.0):
    return I.normal(seed, 91, int(np.prod(shape)), std).reshape(shape)


def _case(ctx, orc, N, d, bf16, seed):
    x = _rand(seed, (N, d), 2.0) + 0.5
    g = 1 + _rand(seed + 1, (d,), 0.1)
    mean = x.mean(axis=1)
    rstd = 1.0 / np.sqrt(x.var(axis=1) + 1e-5)
    xd, gd, md, rd = dev_f32(x), dev_f32(g), dev_f32(mean), dev_f32(rstd)
    dy, dyv = dev_act(_rand(seed + 2, (N, d)), bf16)
    dres = _rand(seed + 3, (N, d))
    dresd = dev_f32(dres)
    outs = []
    for noalloc in (False, True):
        dx = torch.full((N, d), 7.0, device="cuda")
        dxlp = empty_act((N, d), bf16) if bf16 else None
        dg, db, dsum = dev_f32(np.ones(d)), dev_f32(np.ones(d)), dev_f32(np.ones(d))
        common = (DT[bf16], ptr(dy), ptr(xd), ptr(gd), ptr(md), ptr(rd), ptr(dresd), ptr(dx), ptr(dxlp), ptr(dg), ptr(db),
                  ptr(dsum))
        if noalloc:
            ctx.op("layernorm_bwd_noalloc", *common, N, d, 1)
        else:
            ws = torch.empty(pwb.lib().pw_layernorm_bwd_ws_floats(N, d), device="cuda")
            ctx.op("layernorm_bwd", *common, ptr(ws), N, d, 1)
        ctx.synchronize()
        outs.append([host(t) for t in (dx, dg, db, dsum)] + ([host(dxlp)] if bf16 else []))
    for a, b in zip(*outs):
        assert np.array_equal(a, b)                          # the existing entry point, bit for bit
    rdx, rdg, rdb = orc.layernorm_bwd(dyv, x, g)
    dx, dg, db, dsum = outs[1][:4]
    assert_close(dx, rdx + dres, 1e-5)
    assert_close(dg, rdg + 1.0, 1e-5)
    assert_close(db, rdb + 1.0, 1e-5)
    assert_close(dsum, (rdx + dres).sum(axis=0) + 1.0, 1e-5)
    if bf16:
        assert_close(outs[1][4], rdx + dres, 4e-3)


@pytest.mark.parametrize("bf16", [False, True])
def test_layernorm_backward_without_allocation_two_calls_in_a_row(orc, bf16):
    with pwb.Context(0) as ctx:
        _case(ctx, orc, 2100, 2048, bf16, 100)     # 512 blocks of block sums: the array's full extent
        _case(ctx, orc, 37, 256, bf16, 200)        # smaller: stale sums of the first call lie beyond its slots
        _case(ctx, orc, 70, 4096, bf16, 300)       # wide rows (block-per-row kernel) that still fit the array
        # too large for the fixed array: refused, nothing enqueued
        N, d = 600, 4096
        t = torch.zeros((N, d), device="cuda")
        v = torch.zeros(max(N, d), device="cuda")
        dx = torch.full((N, d), 7.0, device="cuda")
        with pytest.raises(pwb.PwError) as e:
            ctx.op("layernorm_bwd_noalloc", pwb.PW_F32, ptr(t), ptr(t), ptr(v), ptr(v), ptr(v), None, ptr(dx), None,
                   ptr(v), ptr(v), None, N, d, 0)
        assert e.value.status == pwb.PW_ERR_UNSUPPORTED
        ctx.synchronize()
        assert (host(dx) == 7.0).all()
