"""The parity criterion of the GPU tests (numpy only, so that the CPU suite can test the criterion itself).

A tensor `got` matches its oracle value `ref` at bar `tol` when BOTH hold:
  * norm:      ||got - ref||_2 / ||ref||_2 < tol                       (the headline error per tensor)
  * elements:  |got_i - ref_i| <= tol * (ELEM_C * rms(ref) + |ref_i|)   for every element i

The norm alone lets a small wrong region hide among millions of good elements (a 16 x 16 block that lost a third of its
contraction contributes a few 1e-3 to the norm of a 4096 x 4096 product); the element bound does not: such a block is
wrong by about half an rms per element, against an allowance of a few hundredths.  The relative term keeps large
elements (the target entry of a row of dlogits is sqrt(V) times the row's rms) from tripping the bound on their own
rounding: tol is never below one bf16 rounding (2^-9) on the bf16 path.  ELEM_C covers the tail of honest rounding
error over up to 1e8 elements plus the elements that are small by cancellation.  rms(ref) is taken over the non-zero
elements of ref: the gradient of an embedding table is zero in the rows of unused ids (nine rows in ten for 1024
tokens over a vocabulary of 8192), and averaging over those zeros would shrink the allowance of the rows that carry
the gradient by the square root of the fill - for dense tensors it is the plain rms.
"""
import os
import sys

import numpy as np

ELEM_C = 8.0

_margins = []          # (name, n, rel_l2 / tol, worst element ratio) of every comparison made in this process


def rel_l2(got, ref):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got))


def elem_ratio(got, ref, tol, extra=None):
    """max_i |got_i - ref_i| / (tol * (ELEM_C * rms(ref) + |ref_i|) + extra_i) and the flat index where it is reached.
    extra: absolute allowance on top (scalar or array), for error that does not come from the path under test - e.g.
    the fp32 storage of a weight, when what is compared is its small update."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    if ref.size == 0:
        return 0.0, -1
    nz = int(np.count_nonzero(ref))
    rms = float(np.sqrt(np.sum(ref * ref) / nz)) if nz else 0.0     # over the support: see the module text
    diff = np.abs(got - ref)
    allow = tol * (ELEM_C * rms + np.abs(ref))
    if extra is not None:
        allow = allow + np.asarray(extra, np.float64)
    if rms == 0.0 and extra is None:                       # an all-zero reference: only exact zeros match element-wise
        i = int(np.argmax(diff))
        return (0.0 if diff.reshape(-1)[i] == 0.0 else np.inf), i
    ratio = diff / allow
    i = int(np.argmax(ratio))
    return float(ratio.reshape(-1)[i]), i


def assert_close(got, ref, tol, name="", norm_slack=0.0, extra=None):
    caller = sys._getframe(1)
    name = f"{caller.f_code.co_name}:{caller.f_lineno}" + (f" {name}" if name != "" else "")
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert got.shape == ref.shape, f"{name}: shape {got.shape} vs oracle {ref.shape}"
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    err = rel_l2(got, ref)
    worst, at = elem_ratio(got, ref, tol, extra)
    _margins.append((name, int(ref.size), err / (tol + norm_slack), worst))
    assert err < tol + norm_slack, f"{name}: relative L2 error {err:.3e} >= {tol + norm_slack:.1e}"
    if worst > 1.0:
        idx = np.unravel_index(at, ref.shape)
        raise AssertionError(f"{name}: element {idx} is {got[idx]!r}, oracle {ref[idx]!r}: |diff| is {worst:.2f}x the "
                             f"allowance tol*({ELEM_C:g}*rms + |ref|) at tol {tol:.1e} (relative L2 of the tensor {err:.3e})")


def dump_margins(path=None):
    """Writes what every comparison of this process used of its two bars (set PW_PARITY_LOG to a file name)."""
    path = path or os.environ.get("PW_PARITY_LOG")
    if not path or not _margins:
        return
    with open(path, "a") as f:
        for name, n, a, b in _margins:
            f.write(f"{name or '-'}\t{n}\t{a:.4f}\t{b:.4f}\n")
