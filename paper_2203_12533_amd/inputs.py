"""Seeded synthetic inputs for the decoder-only LM train step and the dispatch
micro-benchmark.

This module only *draws numbers*: it holds none of the model's arithmetic and
is the one piece of code that both the CPU oracle's tests and the HIP path's
tests/benchmarks use, so both sides start from identical bits.

The paper trains its decoder-only LM (Section 5.3: model dimension 2048,
hidden dimension 8192) on a corpus it does not name; token values do not
change the work of a dense LM step, so uniform seeded tokens with the paper's
model shape stand in for it.

Generator: counter based.  Element ``i`` of tensor ``tid`` under ``seed`` is a
pure function of ``(seed, tid, i)`` through the public splitmix64 finaliser,
so any slice of any tensor can be regenerated on its own, in any order.
Normals come from Box-Muller on two such uniforms.
"""
from __future__ import annotations

from dataclasses import dataclass, asdict, replace
import math
import zlib

import numpy as np

_GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_TID = np.uint64(0xD1342543DE82EF95)
_CHUNK = 1 << 24


def _mix(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function (Steele, Lea, Flood 2014), vectorised."""
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _key(seed: int, tid: int) -> np.uint64:
    with np.errstate(over="ignore"):
        k = np.array([np.uint64(seed & 0xFFFFFFFFFFFFFFFF)], dtype=np.uint64)
        k = _mix(k + _GOLD) ^ (np.uint64(tid) * _TID)
        return _mix(k + _GOLD)[0]


def raw_u64(seed: int, tid: int, start: int, n: int) -> np.ndarray:
    """64 random bits for counters start .. start+n-1 of tensor ``tid``."""
    with np.errstate(over="ignore"):
        idx = np.arange(start, start + n, dtype=np.uint64)
        return _mix(_key(seed, tid) + (idx + np.uint64(1)) * _GOLD)


def uniform01(seed: int, tid: int, n: int, start: int = 0) -> np.ndarray:
    """float64 uniform on [0, 1) with 53 random bits."""
    out = np.empty(n, dtype=np.float64)
    for s in range(0, n, _CHUNK):
        m = min(_CHUNK, n - s)
        out[s:s + m] = (raw_u64(seed, tid, start + s, m) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))
    return out


def normal(seed: int, tid: int, n: int, std: float = 1.0) -> np.ndarray:
    """float32 N(0, std^2): Box-Muller, element i uses counters 2i and 2i+1."""
    out = np.empty(n, dtype=np.float32)
    for s in range(0, n, _CHUNK):
        m = min(_CHUNK, n - s)
        r = raw_u64(seed, tid, 2 * s, 2 * m) >> np.uint64(11)
        u1 = (r[0::2].astype(np.float64) + 1.0) * (1.0 / (1 << 53))   # (0, 1]
        u2 = r[1::2].astype(np.float64) * (1.0 / (1 << 53))           # [0, 1)
        out[s:s + m] = (std * np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)).astype(np.float32)
    return out


def normal_torch(seed: int, tid: int, n: int, std: float, device):
    """The generator of normal() evaluated by torch on `device` (a GPU for the 0.7 G parameters of the measured
    workload, which numpy would take minutes over): the same counters, the same splitmix64 bits (int64 arithmetic
    wraps like uint64; right shifts are made logical by masking), the same Box-Muller formula in float64.  The 64
    random bits are identical to numpy's; log / cos may differ from numpy's in the last place of float64, which the
    rounding to float32 hides for all but a few values in a million."""
    import torch

    def lsr(z, k):                                   # logical shift right of the uint64 held in an int64
        return (z >> k) & ((1 << (64 - k)) - 1)

    def mix(z):
        z = (z ^ lsr(z, 30)) * _i64(_M1)
        z = (z ^ lsr(z, 27)) * _i64(_M2)
        return z ^ lsr(z, 31)

    key, gold = _i64(_key(seed, tid)), _i64(_GOLD)
    out = torch.empty(n, dtype=torch.float32, device=device)
    for s in range(0, n, _CHUNK):
        m = min(_CHUNK, n - s)
        idx = torch.arange(2 * s + 1, 2 * (s + m) + 1, dtype=torch.int64, device=device)
        r = lsr(mix(key + idx * gold), 11)
        u1 = (r[0::2].to(torch.float64) + 1.0) * (1.0 / (1 << 53))
        u2 = r[1::2].to(torch.float64) * (1.0 / (1 << 53))
        out[s:s + m] = (std * torch.sqrt(-2.0 * torch.log(u1)) * torch.cos(2.0 * math.pi * u2)).to(torch.float32)
    return out


def _i64(u) -> int:
    """The int64 with the bit pattern of a uint64."""
    u = int(u)
    return u - (1 << 64) if u >= (1 << 63) else u


def param_torch(cfg, name: str, shape, kind: str, device, seed: int = 1234):
    """One parameter tensor of lm_params / encdec_params (perturb=False), flat float32, drawn on `device`."""
    import torch
    n = int(np.prod(shape))
    if kind == "matrix":
        t = normal_torch(seed, _tid(name), n, cfg.init_std, device)
        return t.to(torch.bfloat16).to(torch.float32) if cfg.bf16 else t      # round-to-nearest-even, as round_to_bf16
    return (torch.ones if kind == "gain" else torch.zeros)(n, dtype=torch.float32, device=device)


def tokens(seed: int, tid: int, shape, vocab: int) -> np.ndarray:
    """int32 token ids uniform over [0, vocab)."""
    n = int(np.prod(shape))
    return (raw_u64(seed, tid, 0, n) % np.uint64(vocab)).astype(np.int32).reshape(shape)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bfloat16 (ties to even); result kept as float32.

    bf16-mode workloads start from bf16-representable weights so that the fp32
    master copy and the bf16 compute copy hold the same numbers at step 0."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def _tid(name: str) -> int:
    return zlib.crc32(name.encode()) & 0x7FFFFFFF


@dataclass(frozen=True)
class LMConfig:
    """Shape of one accelerator's share of the decoder-only LM step."""
    n_layer: int
    d_model: int
    n_head: int
    d_ff: int
    vocab: int
    seq: int
    batch: int
    bf16: bool = False            # False: fp32 everywhere; True: bf16 compute, fp32 master weights
    optimizer: str = "sgd"        # "sgd" | "adam"
    lr: float = 1e-2
    beta1: float = 0.9
    beta2: float = 0.95
    eps: float = 1e-8
    init_std: float = 0.02
    has_embed: bool = True        # False: a pipeline stage fed with activations
    has_head: bool = True         # False: a pipeline stage returning activations
    n_microbatch: int = 1

    @property
    def head_dim(self) -> int:
        return self.d_model // self.n_head

    @property
    def n_tokens(self) -> int:
        return self.batch * self.seq

    def asdict(self):
        return asdict(self)

    def with_(self, **kw) -> "LMConfig":
        return replace(self, **kw)


def workload(name: str) -> LMConfig:
    """The named workloads this build is measured on."""
    if name == "cfg1":   # small fp32 case the CPU oracle finishes in seconds
        return LMConfig(2, 256, 4, 1024, 1024, 128, 4, bf16=False, optimizer="sgd", lr=1e-2)
    if name == "cfg3":   # 12 layers of the paper's 3B-LM layer shape (Section 5.3)
        return LMConfig(12, 2048, 16, 8192, 32768, 1024, 8, bf16=True, optimizer="adam", lr=1e-4)
    if name == "cfg4":   # one stage of a 16-stage pipeline, 8 micro-batches of 1
        return LMConfig(4, 4096, 32, 16384, 0, 2048, 1, bf16=True, optimizer="adam", lr=1e-4,
                        has_embed=False, has_head=False, n_microbatch=8)
    if name == "cfg5":   # wide-layer shard
        return LMConfig(2, 8192, 64, 32768, 32768, 2048, 2, bf16=True, optimizer="adam", lr=1e-4,
                        init_std=0.02 / math.sqrt(2 * 2))
    raise KeyError(name)


def param_shapes(cfg: LMConfig):
    """Ordered (name, shape, kind) list; kind in {"matrix", "bias", "gain"}.

    Linear weights are stored [in, out]; wqkv columns are [Q | K | V], head h
    owning columns h*head_dim .. (h+1)*head_dim of each third."""
    d, F, V, T = cfg.d_model, cfg.d_ff, cfg.vocab, cfg.seq
    out = []
    if cfg.has_embed:
        out += [("wte", (V, d), "matrix"), ("wpe", (T, d), "matrix")]
    for l in range(cfg.n_layer):
        p = f"l{l}."
        out += [(p + "ln1_g", (d,), "gain"), (p + "ln1_b", (d,), "bias"),
                (p + "wqkv", (d, 3 * d), "matrix"), (p + "bqkv", (3 * d,), "bias"),
                (p + "wo", (d, d), "matrix"), (p + "bo", (d,), "bias"),
                (p + "ln2_g", (d,), "gain"), (p + "ln2_b", (d,), "bias"),
                (p + "w1", (d, F), "matrix"), (p + "b1", (F,), "bias"),
                (p + "w2", (F, d), "matrix"), (p + "b2", (d,), "bias")]
    if cfg.has_head:
        out += [("lnf_g", (d,), "gain"), ("lnf_b", (d,), "bias"), ("wh", (d, V), "matrix")]
    return out


def lm_params(cfg: LMConfig, seed: int = 1234, perturb: bool = False) -> dict:
    """Initial parameters.  Matrices and embeddings N(0, init_std); biases 0;
    LayerNorm gain 1.  ``perturb=True`` (tests only) also draws biases
    N(0, init_std) and gains 1 + N(0, init_std) so that mistakes in bias and
    gain handling cannot hide behind zeros and ones.  bf16 configs round every
    value to a bf16-representable one."""
    out = {}
    for name, shape, kind in param_shapes(cfg):
        n = int(np.prod(shape))
        if kind == "matrix":
            a = normal(seed, _tid(name), n, cfg.init_std)
        elif kind == "bias":
            a = normal(seed, _tid(name), n, cfg.init_std) if perturb else np.zeros(n, np.float32)
        else:
            a = np.ones(n, np.float32)
            if perturb:
                a = a + normal(seed, _tid(name), n, cfg.init_std)
        if cfg.bf16:
            a = round_to_bf16(a)
        out[name] = a.reshape(shape)
    return out


def lm_tokens(cfg: LMConfig, seed: int = 1234) -> np.ndarray:
    """[batch, seq+1] ids: inputs are columns 0..seq-1, targets columns 1..seq."""
    return tokens(seed, _tid("tokens"), (cfg.batch, cfg.seq + 1), cfg.vocab)


def stage_io(cfg: LMConfig, seed: int = 1234):
    """Pipeline-stage inputs X_mb and output-gradients dY_mb, N(0,1), one pair per micro-batch."""
    n = cfg.n_tokens * cfg.d_model
    xs, dys = [], []
    for mb in range(cfg.n_microbatch):
        x = normal(seed, _tid(f"stage_x{mb}"), n, 1.0)
        dy = normal(seed, _tid(f"stage_dy{mb}"), n, 1.0)
        if cfg.bf16:
            x, dy = round_to_bf16(x), round_to_bf16(dy)
        xs.append(x.reshape(cfg.n_tokens, cfg.d_model))
        dys.append(dy.reshape(cfg.n_tokens, cfg.d_model))
    return xs, dys


@dataclass(frozen=True)
class EncDecConfig:
    """Shape of one accelerator's share of the encoder-decoder step (the text-to-text family of the paper's
    Table 1, built from the decoder-only model's pieces)."""
    n_enc_layer: int
    n_dec_layer: int
    d_model: int
    n_head: int
    d_ff: int
    vocab: int
    src_len: int
    tgt_len: int
    batch: int
    bf16: bool = False
    optimizer: str = "sgd"
    lr: float = 1e-2
    beta1: float = 0.9
    beta2: float = 0.95
    eps: float = 1e-8
    init_std: float = 0.02

    @property
    def head_dim(self) -> int:
        return self.d_model // self.n_head

    @property
    def n_tokens(self) -> int:
        """Source plus target positions of one step."""
        return self.batch * (self.src_len + self.tgt_len)

    def with_(self, **kw) -> "EncDecConfig":
        return replace(self, **kw)


def encdec_workload(name: str) -> EncDecConfig:
    if name == "ed1":    # small fp32 case the CPU oracle finishes in seconds; ragged lengths
        return EncDecConfig(2, 2, 256, 4, 1024, 1024, 96, 80, 3, bf16=False, optimizer="sgd", lr=1e-2)
    if name == "ed3":    # 6 + 6 layers of the cfg3 layer shape, 1024 source and 1024 target positions
        return EncDecConfig(6, 6, 2048, 16, 8192, 32768, 1024, 1024, 8, bf16=True, optimizer="adam", lr=1e-4)
    raise KeyError(name)


def encdec_param_shapes(cfg: EncDecConfig):
    """Ordered (name, shape, kind) list.  Linear weights are [in, out]; wqkv columns are [Q | K | V], wkv
    columns [K | V]; head h owns columns h*head_dim .. (h+1)*head_dim of each part."""
    d, F, V = cfg.d_model, cfg.d_ff, cfg.vocab

    def attn(p):
        return [(p + "ln1_g", (d,), "gain"), (p + "ln1_b", (d,), "bias"),
                (p + "wqkv", (d, 3 * d), "matrix"), (p + "bqkv", (3 * d,), "bias"),
                (p + "wo", (d, d), "matrix"), (p + "bo", (d,), "bias")]

    def ffn(p):
        return [(p + "ln2_g", (d,), "gain"), (p + "ln2_b", (d,), "bias"),
                (p + "w1", (d, F), "matrix"), (p + "b1", (F,), "bias"),
                (p + "w2", (F, d), "matrix"), (p + "b2", (d,), "bias")]

    out = [("enc.wte", (V, d), "matrix"), ("enc.wpe", (cfg.src_len, d), "matrix")]
    for l in range(cfg.n_enc_layer):
        out += attn(f"e{l}.") + ffn(f"e{l}.")
    out += [("enc.lnf_g", (d,), "gain"), ("enc.lnf_b", (d,), "bias"),
            ("dec.wte", (V, d), "matrix"), ("dec.wpe", (cfg.tgt_len, d), "matrix")]
    for l in range(cfg.n_dec_layer):
        p = f"d{l}."
        out += attn(p)
        out += [(p + "lnx_g", (d,), "gain"), (p + "lnx_b", (d,), "bias"),
                (p + "wq", (d, d), "matrix"), (p + "bq", (d,), "bias"),
                (p + "wkv", (d, 2 * d), "matrix"), (p + "bkv", (2 * d,), "bias"),
                (p + "wox", (d, d), "matrix"), (p + "box", (d,), "bias")]
        out += ffn(p)
    out += [("dec.lnf_g", (d,), "gain"), ("dec.lnf_b", (d,), "bias"), ("wh", (d, V), "matrix")]
    return out


def encdec_params(cfg: EncDecConfig, seed: int = 1234, perturb: bool = False) -> dict:
    """Initial parameters, drawn like lm_params."""
    out = {}
    for name, shape, kind in encdec_param_shapes(cfg):
        n = int(np.prod(shape))
        if kind == "matrix":
            a = normal(seed, _tid(name), n, cfg.init_std)
        elif kind == "bias":
            a = normal(seed, _tid(name), n, cfg.init_std) if perturb else np.zeros(n, np.float32)
        else:
            a = np.ones(n, np.float32)
            if perturb:
                a = a + normal(seed, _tid(name), n, cfg.init_std)
        if cfg.bf16:
            a = round_to_bf16(a)
        out[name] = a.reshape(shape)
    return out


def encdec_tokens(cfg: EncDecConfig, seed: int = 1234):
    """(src [batch, src_len], tgt [batch, tgt_len+1]): decoder inputs are tgt columns 0..tgt_len-1, targets
    columns 1..tgt_len."""
    return (tokens(seed, _tid("src_tokens"), (cfg.batch, cfg.src_len), cfg.vocab),
            tokens(seed, _tid("tgt_tokens"), (cfg.batch, cfg.tgt_len + 1), cfg.vocab))


def dispatch_input(seed: int = 1234, n: int = 128) -> np.ndarray:
    """x for the dispatch micro-benchmark: fp32 uniform [0, 1)."""
    r = raw_u64(seed, _tid("dispatch_x"), 0, n) >> np.uint64(40)      # 24 bits: exact in fp32, < 1
    return (r.astype(np.float64) * (1.0 / (1 << 24))).astype(np.float32)
