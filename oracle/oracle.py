"""ctypes wrapper of the CPU oracle (``liboracle.so``, built from oracle/*.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of bench.py.  It never imports the HIP package
and the HIP package never imports it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import sys
import time

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with g++ (plain loops, OpenMP over independent iterations)."""
    srcs = [os.path.join(_HERE, "oracle_capi.cpp")]
    deps = srcs + [os.path.join(_HERE, h) for h in ("lm_oracle.hpp", "encdec_oracle.hpp")]
    if not force and os.path.exists(_SO) and all(os.path.getmtime(_SO) >= os.path.getmtime(f) for f in deps):
        return _SO
    cmd = ["g++", "-O3", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared", "-std=c++17",
           "-fno-fast-math", "-o", _SO] + srcs
    subprocess.check_call(cmd)
    return _SO


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build()
        _lib = C.CDLL(_SO)
        _lib.orc_lm_param_count.restype = C.c_int64
        _lib.orc_lm_param_total.restype = C.c_int64
        _lib.orc_encdec_param_count.restype = C.c_int64
        _lib.orc_encdec_param_total.restype = C.c_int64
    return _lib


class Shape(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("L", "d", "H", "F", "V", "T", "B", "has_embed", "has_head")]


class Opt(C.Structure):
    _fields_ = [("kind", C.c_int), ("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double),
                ("eps", C.c_double), ("t", C.c_int)]


def _shape(cfg) -> Shape:
    return Shape(cfg.n_layer, cfg.d_model, cfg.n_head, cfg.d_ff, cfg.vocab, cfg.seq, cfg.batch,
                 int(cfg.has_embed), int(cfg.has_head))


def _opt(cfg, t: int, update: bool) -> Opt:
    kind = 0 if not update else {"sgd": 1, "adam": 2}[cfg.optimizer]
    return Opt(kind, cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, t)


def _p(a, ty=C.c_double):
    return None if a is None else a.ctypes.data_as(C.POINTER(ty))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def threads() -> int:
    return lib().orc_threads()


# ---- single operations (double precision) -------------------------------------------------------

def embedding_fwd(inp, wte, wpe):
    inp, wte, wpe = _i32(inp), _f64(wte), _f64(wpe)
    B, T = inp.shape
    d = wte.shape[1]
    x = np.empty((B * T, d))
    lib().orc_embedding_fwd(_p(inp, C.c_int32), _p(wte), _p(wpe), _p(x), B, T, d)
    return x


def embedding_bwd(inp, dx, V):
    inp, dx = _i32(inp), _f64(dx)
    B, T = inp.shape
    d = dx.shape[-1]
    dwte, dwpe = np.empty((V, d)), np.empty((T, d))
    lib().orc_embedding_bwd(_p(inp, C.c_int32), _p(dx), _p(dwte), _p(dwpe), B, T, d, V)
    return dwte, dwpe


def layernorm_fwd(x, g, b):
    x, g, b = _f64(x), _f64(g), _f64(b)
    N, d = x.shape
    y, mean, rstd = np.empty((N, d)), np.empty(N), np.empty(N)
    lib().orc_layernorm_fwd(_p(x), _p(g), _p(b), _p(y), _p(mean), _p(rstd), N, d)
    return y, mean, rstd


def layernorm_bwd(dy, x, g):
    dy, x, g = _f64(dy), _f64(x), _f64(g)
    N, d = x.shape
    dx, dg, db = np.empty((N, d)), np.empty(d), np.empty(d)
    lib().orc_layernorm_bwd(_p(dy), _p(x), _p(g), _p(dx), _p(dg), _p(db), N, d)
    return dx, dg, db


def linear_fwd(x, W, b=None):
    x, W = _f64(x), _f64(W)
    b = None if b is None else _f64(b)
    N, i = x.shape
    o = W.shape[1]
    y = np.empty((N, o))
    lib().orc_linear_fwd(_p(x), _p(W), _p(b), _p(y), N, i, o)
    return y


def linear_bwd(x, W, dy):
    x, W, dy = _f64(x), _f64(W), _f64(dy)
    N, i = x.shape
    o = W.shape[1]
    dx, dW, db = np.empty((N, i)), np.empty((i, o)), np.empty(o)
    lib().orc_linear_bwd(_p(x), _p(W), _p(dy), _p(dx), _p(dW), _p(db), N, i, o)
    return dx, dW, db


def gelu_fwd(u):
    u = _f64(u)
    h = np.empty_like(u)
    lib().orc_gelu_fwd(_p(u), _p(h), C.c_int64(u.size))
    return h


def gelu_bwd(u, dh):
    u, dh = _f64(u), _f64(dh)
    du = np.empty_like(u)
    lib().orc_gelu_bwd(_p(u), _p(dh), _p(du), C.c_int64(u.size))
    return du


def attention_fwd(qkv, B, T, H, hd, want_probs=False):
    qkv = _f64(qkv)
    o = np.empty((B * T, H * hd))
    probs = np.empty((B, H, T, T)) if want_probs else None
    lib().orc_attention_fwd(_p(qkv), _p(o), _p(probs), B, T, H, hd)
    return (o, probs) if want_probs else o


def attention_bwd(qkv, dout, B, T, H, hd):
    qkv, dout = _f64(qkv), _f64(dout)
    dqkv = np.empty_like(qkv)
    lib().orc_attention_bwd(_p(qkv), _p(dout), _p(dqkv), B, T, H, hd)
    return dqkv


def softmax_xent(z, tgt, want_grad=True):
    z, tgt = _f64(z), _i32(tgt)
    N, V = z.shape
    loss = C.c_double()
    dz = np.empty((N, V)) if want_grad else None
    lib().orc_softmax_xent(_p(z), _p(tgt, C.c_int32), N, V, C.byref(loss), _p(dz))
    return (loss.value, dz) if want_grad else loss.value


def sgd(w, g, lr):
    w, g = _f64(w).copy(), _f64(g)
    lib().orc_sgd(_p(w), _p(g), C.c_int64(w.size), C.c_double(lr))
    return w


def adam(w, m, v, g, lr, b1, b2, eps, t):
    w, m, v, g = _f64(w).copy(), _f64(m).copy(), _f64(v).copy(), _f64(g)
    lib().orc_adam(_p(w), _p(m), _p(v), _p(g), C.c_int64(w.size), C.c_double(lr), C.c_double(b1),
                   C.c_double(b2), C.c_double(eps), t)
    return w, m, v


# ---- whole step ---------------------------------------------------------------------------------

def param_table(cfg):
    """[(name, offset, numel)] of the oracle's own flat parameter layout."""
    s = _shape(cfg)
    out = []
    name = C.create_string_buffer(64)
    off, num = C.c_int64(), C.c_int64()
    for i in range(lib().orc_lm_param_count(C.byref(s))):
        lib().orc_lm_param_info(C.byref(s), C.c_int64(i), name, 64, C.byref(off), C.byref(num))
        out.append((name.value.decode(), off.value, num.value))
    return out


def pack(cfg, params: dict, dtype=np.float64) -> np.ndarray:
    s = _shape(cfg)
    flat = np.zeros(lib().orc_lm_param_total(C.byref(s)), dtype=dtype)
    for name, off, num in param_table(cfg):
        flat[off:off + num] = np.asarray(params[name], dtype=dtype).reshape(-1)
    return flat


def unpack(cfg, flat: np.ndarray, like: dict) -> dict:
    return {name: flat[off:off + num].reshape(like[name].shape).copy() for name, off, num in param_table(cfg)}


def lm_train_step(cfg, params: dict, tokens, state=None, t: int = 1, update: bool = True,
                  want_logits: bool = False, backward: bool = True, dtype=np.float64):
    """One train step.  Returns dict(loss, grads, params, m, v[, logits]).

    ``dtype=np.float32`` runs the single-precision instantiation (used only to
    show the oracle's own rounding is far below the fp32 parity tolerance)."""
    ty = C.c_double if dtype == np.float64 else C.c_float
    s = _shape(cfg)
    P = pack(cfg, params, dtype)
    if state is None:
        M, V = np.zeros_like(P), np.zeros_like(P)
    else:
        M, V = pack(cfg, state["m"], dtype), pack(cfg, state["v"], dtype)
    G = np.zeros_like(P)
    tok = _i32(tokens)
    logits = np.empty((cfg.n_tokens, cfg.vocab), dtype=dtype) if want_logits else None
    loss = ty()
    o = _opt(cfg, t, update and backward)
    fn = lib().orc_lm_train_step if dtype == np.float64 else lib().orc_lm_train_step_f32
    t0 = time.perf_counter()
    rc = fn(C.byref(s), _p(P, ty), _p(M, ty), _p(V, ty), _p(tok, C.c_int32), C.byref(o), C.byref(loss),
            _p(G, ty), _p(logits, ty), int(backward))
    seconds = time.perf_counter() - t0
    if rc:
        raise RuntimeError("oracle lm_train_step rejected the configuration")
    out = {"loss": float(loss.value), "seconds": seconds}   # time inside the C++ step only
    if backward:
        out.update(grads=unpack(cfg, G, params), params=unpack(cfg, P, params),
                   m=unpack(cfg, M, params), v=unpack(cfg, V, params))
    if want_logits:
        out["logits"] = logits
    return out


def time_train_step(cfg, seed: int = 0) -> float:
    """Seconds the C++ oracle takes for one full train step of `cfg` on freshly drawn weights
    (numpy's own generator: the values only have to be ordinary numbers, nothing is compared)."""
    s = _shape(cfg)
    total = lib().orc_lm_param_total(C.byref(s))
    rng = np.random.default_rng(seed)
    P = rng.standard_normal(total) * cfg.init_std
    M, V, G = np.zeros(total), np.zeros(total), np.zeros(total)
    tok = rng.integers(0, cfg.vocab, size=(cfg.batch, cfg.seq + 1)).astype(np.int32)
    loss = C.c_double()
    o = _opt(cfg, 1, True)
    t0 = time.perf_counter()
    rc = lib().orc_lm_train_step(C.byref(s), _p(P), _p(M), _p(V), _p(tok, C.c_int32), C.byref(o), C.byref(loss),
                                 _p(G), None, 1)
    dt = time.perf_counter() - t0
    if rc or not np.isfinite(loss.value):
        raise RuntimeError("oracle step failed")
    return dt


def stage_fwd_bwd(cfg, params: dict, xs, dys):
    """GPipe-like schedule on one pipeline stage: returns (Y list, dX list, grads dict)."""
    s = _shape(cfg)
    P = pack(cfg, params)
    n_mb = len(xs)
    X = _f64(np.stack(xs))
    dY = _f64(np.stack(dys))
    Y, dX, G = np.empty_like(X), np.empty_like(X), np.zeros_like(P)
    rc = lib().orc_stage_fwd_bwd(C.byref(s), _p(P), n_mb, _p(X), _p(dY), _p(Y), _p(dX), _p(G))
    if rc:
        raise RuntimeError("oracle stage_fwd_bwd rejected the configuration")
    return list(Y), list(dX), unpack(cfg, G, params)


# ---- encoder-decoder workload -------------------------------------------------------------------

def mha_fwd(q, k, v, B, Tq, Tk, H, hd, causal=False):
    """Multi-head attention of Tq queries over Tk keys.  q [B*Tq, >= H*hd], k and v [B*Tk, >= H*hd] may be
    column slices of wider arrays (k and v of the same one): rows are taken at their strides."""
    q, k, v, ldq, ldkv = _strided(q, k, v)
    o = np.empty((B * Tq, H * hd))
    rc = lib().orc_mha_fwd(q, C.c_int64(ldq), k, v, C.c_int64(ldkv), _p(o), B, Tq, Tk, H, hd, int(causal))
    if rc:
        raise ValueError("causal attention needs Tq == Tk")
    return o


def mha_bwd(q, k, v, dout, B, Tq, Tk, H, hd, causal=False):
    """Returns (dq [B*Tq, H*hd], dk [B*Tk, H*hd], dv [B*Tk, H*hd])."""
    q, k, v, ldq, ldkv = _strided(q, k, v)
    dout = _f64(dout)
    d = H * hd
    dq, dk, dv = np.empty((B * Tq, d)), np.empty((B * Tk, d)), np.empty((B * Tk, d))
    rc = lib().orc_mha_bwd(q, C.c_int64(ldq), k, v, C.c_int64(ldkv), _p(dout), _p(dq), C.c_int64(d), _p(dk), _p(dv),
                           C.c_int64(d), B, Tq, Tk, H, hd, int(causal))
    if rc:
        raise ValueError("causal attention needs Tq == Tk")
    return dq, dk, dv


_keep = []


def _strided(q, k, v):
    """Pointers and row strides of 2-D float64 arrays that may be column slices of C-contiguous parents."""
    out = []
    for a in (q, k, v):
        a = np.asarray(a)
        if a.dtype != np.float64 or a.ndim != 2 or a.strides[1] != 8:
            a = _f64(a)
        out.append(a)
    q, k, v = out
    if k.strides[0] != v.strides[0]:
        k, v = _f64(k), _f64(v)
    _keep[:] = [q, k, v]   # alive until the next call returns
    cast = lambda a: C.cast(a.ctypes.data, C.POINTER(C.c_double))
    return cast(q), cast(k), cast(v), q.strides[0] // 8, k.strides[0] // 8


class EncDecShape(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("Le", "Ld", "d", "H", "F", "V", "Ts", "Tt", "B")]


def _ed_shape(cfg) -> EncDecShape:
    return EncDecShape(cfg.n_enc_layer, cfg.n_dec_layer, cfg.d_model, cfg.n_head, cfg.d_ff, cfg.vocab, cfg.src_len,
                       cfg.tgt_len, cfg.batch)


def encdec_param_table(cfg):
    s = _ed_shape(cfg)
    out = []
    name = C.create_string_buffer(64)
    off, num = C.c_int64(), C.c_int64()
    for i in range(lib().orc_encdec_param_count(C.byref(s))):
        lib().orc_encdec_param_info(C.byref(s), C.c_int64(i), name, 64, C.byref(off), C.byref(num))
        out.append((name.value.decode(), off.value, num.value))
    return out


def encdec_train_step(cfg, params: dict, src, tgt, state=None, t: int = 1, update: bool = True,
                      want_logits: bool = False, backward: bool = True):
    """One encoder-decoder train step in double.  Returns dict(loss, grads, params, m, v[, logits])."""
    s = _ed_shape(cfg)
    tab = encdec_param_table(cfg)
    total = lib().orc_encdec_param_total(C.byref(s))

    def pk(dct):
        flat = np.zeros(total)
        for name, off, num in tab:
            flat[off:off + num] = np.asarray(dct[name], dtype=np.float64).reshape(-1)
        return flat

    def unpk(flat):
        return {name: flat[off:off + num].reshape(np.shape(params[name])).copy() for name, off, num in tab}

    P = pk(params)
    M, V = (np.zeros_like(P), np.zeros_like(P)) if state is None else (pk(state["m"]), pk(state["v"]))
    G = np.zeros_like(P)
    src, tgt = _i32(src), _i32(tgt)
    logits = np.empty((cfg.batch * cfg.tgt_len, cfg.vocab)) if want_logits else None
    loss = C.c_double()
    o = _opt(cfg, t, update and backward)
    t0 = time.perf_counter()
    rc = lib().orc_encdec_train_step(C.byref(s), _p(P), _p(M), _p(V), _p(src, C.c_int32), _p(tgt, C.c_int32),
                                     C.byref(o), C.byref(loss), _p(G), _p(logits), int(backward))
    seconds = time.perf_counter() - t0
    if rc:
        raise RuntimeError("oracle encdec_train_step rejected the configuration")
    out = {"loss": float(loss.value), "seconds": seconds}
    if backward:
        out.update(grads=unpk(G), params=unpk(P), m=unpk(M), v=unpk(V))
    if want_logits:
        out["logits"] = logits
    return out


# ---- dispatch micro-benchmark -------------------------------------------------------------------

def chain_add(x, L: int, c: float = 1.0):
    x = np.ascontiguousarray(x, dtype=np.float32)
    y = np.empty_like(x)
    lib().orc_chain_add_f32(_p(x, C.c_float), _p(y, C.c_float), x.size, L, C.c_float(c))
    return y


def scalar_fn(kind: str, x, c: float):
    x = np.ascontiguousarray(x, dtype=np.float32)
    y = np.empty_like(x)
    k = {"mul": 0, "add": 1, "div": 2}[kind]
    lib().orc_scalar_fn_f32(k, _p(x, C.c_float), _p(y, C.c_float), x.size, C.c_float(c))
    return y


if __name__ == "__main__":
    print(build())
    sys.exit(0)
