"""The parity criterion itself (tests/parity.py), on the CPU: honest rounding passes, a small wrong region that the
norm alone would let through does not."""
import numpy as np
import pytest

from paper_2203_12533_amd import inputs as I
from parity import ELEM_C, assert_close, elem_ratio, rel_l2


def _product(M=1024, N=1024, K=192, seed=3):
    rng = np.random.default_rng(seed)
    a = I.round_to_bf16(rng.standard_normal((M, K)).astype(np.float32)).astype(np.float64)
    b = I.round_to_bf16((0.05 * rng.standard_normal((K, N))).astype(np.float32)).astype(np.float64)
    return a, b, a @ b


def test_honest_bf16_rounding_passes_both_bars():
    _, _, c = _product()
    got = I.round_to_bf16(c.astype(np.float32)).astype(np.float64)      # the only error a correct bf16 kernel must have
    assert_close(got, c, 4e-3)
    worst, _ = elem_ratio(got, c, 4e-3)
    assert worst < 0.6                                                    # 2^-9 |c| against 4e-3 (8 rms + |c|)


def test_a_block_that_lost_one_k_tile_passes_the_norm_and_fails_the_element_bar():
    a, b, c = _product(4096, 4096)                                          # the shape of the GPU test it guards
    got = I.round_to_bf16(c.astype(np.float32)).astype(np.float64)
    # one 16 x 16 accumulator block computed without the last of its three 64-deep k-tiles
    got[512:528, 256:272] = a[512:528, :128] @ b[:128, 256:272]
    assert rel_l2(got, c) < 4e-3                                          # the norm alone does not see it
    with pytest.raises(AssertionError, match="element"):
        assert_close(got, c, 4e-3)
    # and at the end-to-end bar a single wrong 16 x 16 block of a gradient still shows
    assert rel_l2(got, c) < 2e-2
    with pytest.raises(AssertionError, match="element"):
        assert_close(got, c, 2e-2)


def test_one_wrong_element_and_one_swapped_pair_fail():
    _, _, c = _product(256, 256, 64)
    got = c.copy()
    got[10, 20] = -got[10, 20] if abs(got[10, 20]) > 0.1 else got[10, 20] + 1.0   # a sign flip
    with pytest.raises(AssertionError):
        assert_close(got, c, 2e-2)
    got = c.copy()
    got[[5, 6]] = got[[6, 5]]                                              # two rows exchanged
    with pytest.raises(AssertionError):
        assert_close(got, c, 2e-2)


def test_heavy_tailed_rows_and_exact_zeros():
    # a row of dlogits: one entry sqrt(V) times the rms of the row; its own bf16 rounding must not trip the bound
    V = 32768
    p = np.full(V, 1.0 / V)
    dz = p.copy()
    dz[123] -= 1.0
    got = I.round_to_bf16(dz.astype(np.float32)).astype(np.float64)
    assert_close(got, dz, 6e-3)
    # all-zero reference (rows of unused ids in the embedding gradient): only exact zeros match
    assert_close(np.zeros(7), np.zeros(7), 1e-5)
    with pytest.raises(AssertionError):
        assert_close(np.full(7, 1e-30), np.zeros(7), 1e-5)
    with pytest.raises(AssertionError, match="shape"):
        assert_close(np.zeros((2, 3)), np.zeros((3, 2)), 1e-5)
    with pytest.raises(AssertionError, match="non-finite"):
        assert_close(np.array([1.0, np.nan]), np.array([1.0, 1.0]), 1e-5)
    assert ELEM_C == 8.0


def test_rows_of_zeros_do_not_shrink_the_allowance_of_the_rows_that_carry_values():
    """An embedding gradient: most rows exactly zero.  The same honest error on the used rows must use the same share
    of the allowance whether the zero rows are there or not."""
    rng = np.random.default_rng(5)
    dense = rng.standard_normal((64, 256))
    err = 2e-3 * rng.standard_normal((64, 256))
    sparse, sparse_err = np.zeros((1024, 256)), np.zeros((1024, 256))
    rows = rng.choice(1024, 64, replace=False)
    sparse[rows], sparse_err[rows] = dense, err
    a, _ = elem_ratio(dense + err, dense, 2e-2)
    b, _ = elem_ratio(sparse + sparse_err, sparse, 2e-2)
    assert a == pytest.approx(b, rel=1e-12)
    assert_close(sparse + sparse_err, sparse, 2e-2)
