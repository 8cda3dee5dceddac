"""Thin ctypes binding of libpw.so (include/pw.h): argument marshalling only.

Every step of the hot path runs in the library's HIP kernels.  PyTorch is used
by callers for device memory and streams; this module only needs raw device
pointers (``tensor.data_ptr()``).  If the library is missing the import of any
symbol fails loudly: there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpw.so")

PW_OK, PW_ERR_INVALID, PW_ERR_SHAPE, PW_ERR_DTYPE, PW_ERR_OOM, PW_ERR_DEVICE, PW_ERR_NOT_READY, \
    PW_ERR_POISONED, PW_ERR_UNSUPPORTED = range(9)
STATUS_NAMES = ["PW_OK", "PW_ERR_INVALID", "PW_ERR_SHAPE", "PW_ERR_DTYPE", "PW_ERR_OOM", "PW_ERR_DEVICE",
                "PW_ERR_NOT_READY", "PW_ERR_POISONED", "PW_ERR_UNSUPPORTED"]
PW_F32, PW_BF16, PW_I32 = 0, 1, 2
PW_FN_ADD_CONST, PW_FN_MUL_CONST, PW_FN_DIV_CONST, PW_FN_BUSY, PW_FN_BUSY_CHAIN, PW_FN_ADD2 = 1, 2, 3, 4, 5, 6
PW_DISPATCH_PARALLEL, PW_DISPATCH_SEQUENTIAL = 0, 1
PW_SCHED_FIFO, PW_SCHED_PROPORTIONAL = 0, 1
PW_FN_LM_TRAIN_STEP, PW_FN_STAGE_FWD, PW_FN_STAGE_BWD, PW_FN_ENCDEC_TRAIN_STEP = 16, 17, 18, 19
PW_STREAM, PW_GRAPH, PW_SEQUENTIAL = 0, 1, 2
PW_PARAMS, PW_GRADS, PW_ADAM_M, PW_ADAM_V = 0, 1, 2, 3
PW_EPI_STORE, PW_EPI_BIAS, PW_EPI_BIAS_RESIDUAL, PW_EPI_BIAS_GELU, PW_EPI_GELU_BWD, PW_EPI_ADAM, PW_EPI_XENT_STATS, \
    PW_EPI_XENT_GRAD = range(8)


class TensorSpec(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("rank", C.c_int32), ("dims", C.c_int64 * 4)]


class FnDesc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("n_in", C.c_int32), ("n_out", C.c_int32),
                ("in_", TensorSpec * 8), ("out", TensorSpec * 8),
                ("params", C.c_void_p), ("params_bytes", C.c_size_t)]


class StageParams(C.Structure):
    _fields_ = [("model", C.c_void_p), ("microbatch", C.c_int32)]


class LMConfigC(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layer", "d_model", "n_head", "d_ff", "vocab", "seq", "batch", "bf16",
                                         "optimizer")] + \
               [(n, C.c_float) for n in ("lr", "beta1", "beta2", "eps")] + \
               [(n, C.c_int32) for n in ("has_embed", "has_head", "n_microbatch", "fused_update", "fused_head_loss")]


class AdamEpilogue(C.Structure):
    _fields_ = [("w", C.c_void_p), ("m", C.c_void_p), ("v", C.c_void_p), ("w_bf16", C.c_void_p),
                ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float), ("t", C.c_int32)]


class XentEpilogue(C.Structure):
    _fields_ = [("tokens", C.c_void_p), ("T", C.c_int32), ("part", C.c_void_p), ("zt", C.c_void_p),
                ("lse", C.c_void_p), ("inv_n", C.c_float)]


class GemmShapeRow(C.Structure):
    _fields_ = [("M", C.c_int64), ("N", C.c_int64), ("K", C.c_int64), ("a_kmajor", C.c_int32), ("b_kmajor", C.c_int32),
                ("epilogue", C.c_int32), ("members", C.c_int32), ("launches", C.c_int64), ("total_ms", C.c_double),
                ("total_flops", C.c_double)]


class GemmArgs(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("a_kmajor", C.c_int32), ("b_kmajor", C.c_int32),
                ("M", C.c_int64), ("N", C.c_int64), ("K", C.c_int64),
                ("lda", C.c_int64), ("ldb", C.c_int64), ("ldc", C.c_int64),
                ("epilogue", C.c_int32), ("out_dtype", C.c_int32), ("accumulate", C.c_int32),
                ("A", C.c_void_p), ("B", C.c_void_p), ("bias", C.c_void_p), ("aux", C.c_void_p),
                ("C", C.c_void_p), ("C2", C.c_void_p), ("b_colsum", C.c_void_p),
                ("adam", C.POINTER(AdamEpilogue)), ("xent", C.POINTER(XentEpilogue))]


class EncDecConfigC(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_enc_layer", "n_dec_layer", "d_model", "n_head", "d_ff", "vocab", "src_len",
                                         "tgt_len", "batch", "bf16", "optimizer")] + \
               [(n, C.c_float) for n in ("lr", "beta1", "beta2", "eps")] + [("fused_update", C.c_int32)]


class MhaArgs(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("q", C.c_void_p), ("k", C.c_void_p), ("v", C.c_void_p),
                ("ldq", C.c_int64), ("ldkv", C.c_int64),
                ("B", C.c_int32), ("Tq", C.c_int32), ("Tk", C.c_int32), ("H", C.c_int32), ("hd", C.c_int32),
                ("causal", C.c_int32)]


class PwError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else status}: {msg}")
        self.status = status


_lib = None

# name -> (restype, argtypes); everything pw.h declares
_SIGS = {
    "pw_ctx_create": (C.c_int, [C.c_int, C.c_void_p, C.POINTER(C.c_void_p)]),
    "pw_ctx_destroy": (C.c_int, [C.c_void_p]),
    "pw_last_error": (C.c_char_p, [C.c_void_p]),
    "pw_ctx_stream": (C.c_void_p, [C.c_void_p]),
    "pw_ctx_synchronize": (C.c_int, [C.c_void_p]),
    "pw_ctx_set_gate_timeout_ms": (C.c_int, [C.c_void_p, C.c_int]),
    "pw_ctx_stats": (C.c_int, [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]),
    "pw_compile_fn": (C.c_int, [C.c_void_p, C.POINTER(FnDesc), C.POINTER(C.c_uint64)]),
    "pw_fn_release": (C.c_int, [C.c_void_p, C.c_uint64]),
    "pw_run_fn": (C.c_int, [C.c_void_p, C.c_uint64, C.POINTER(C.c_uint64), C.c_int, C.POINTER(C.c_uint64), C.c_int]),
    "pw_chain": (C.c_int, [C.c_void_p, C.POINTER(C.c_uint64), C.c_int, C.POINTER(C.c_uint64), C.c_int,
                           C.POINTER(C.c_uint64), C.c_int, C.c_int]),
    "pw_train_step": (C.c_int, [C.c_void_p, C.c_uint64, C.c_uint64, C.POINTER(C.c_uint64)]),
    "pw_ctx_set_owner": (C.c_int, [C.c_void_p, C.c_uint64]),
    "pw_owner_collect": (C.c_int, [C.c_void_p, C.c_uint64, C.POINTER(C.c_int64)]),
    "pw_ctx_set_memory_limit": (C.c_int, [C.c_void_p, C.c_int64]),
    "pw_sched_client_fail": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_int64)]),
    "pw_sched_stalls": (C.c_int, [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_double)]),
    "pw_program_create": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.POINTER(C.c_int32), C.c_int,
                                    C.POINTER(C.c_void_p)]),
    "pw_program_run": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(C.c_uint64), C.c_int, C.POINTER(C.c_uint64), C.c_int, C.c_int]),
    "pw_program_destroy": (C.c_int, [C.c_void_p]),
    "pw_sched_create": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_void_p)]),
    "pw_sched_destroy": (C.c_int, [C.c_void_p]),
    "pw_sched_add_client": (C.c_int, [C.c_void_p, C.c_double, C.POINTER(C.c_int)]),
    "pw_sched_submit": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_uint64), C.c_int, C.c_uint64, C.POINTER(C.c_uint64)]),
    "pw_sched_wait": (C.c_int, [C.c_void_p, C.c_uint64, C.c_void_p, C.c_size_t]),
    "pw_sched_drain": (C.c_int, [C.c_void_p]),
    "pw_sched_client_stats": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_double)]),
    "pw_sched_trace": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.POINTER(C.c_int)]),
    "pw_ctx_set_executors": (C.c_int, [C.c_void_p, C.c_int]),
    "pw_ctx_set_executor_prep_us": (C.c_int, [C.c_void_p, C.c_int]),
    "pw_pipeline": (C.c_int, [C.c_void_p, C.POINTER(C.c_uint64), C.POINTER(C.c_int32), C.c_int, C.c_uint64,
                              C.POINTER(C.c_uint64), C.c_int]),
    "pw_await": (C.c_int, [C.c_void_p, C.c_uint64, C.c_void_p, C.c_size_t]),
    "pw_future_from_host": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(TensorSpec), C.POINTER(C.c_uint64)]),
    "pw_future_wrap_device": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(TensorSpec), C.POINTER(C.c_uint64)]),
    "pw_future_pending": (C.c_int, [C.c_void_p, C.POINTER(TensorSpec), C.POINTER(C.c_uint64)]),
    "pw_future_resolve": (C.c_int, [C.c_void_p, C.c_uint64, C.c_void_p]),
    "pw_future_query": (C.c_int, [C.c_void_p, C.c_uint64]),
    "pw_future_spec": (C.c_int, [C.c_void_p, C.c_uint64, C.POINTER(TensorSpec)]),
    "pw_future_device_ptr": (C.c_int, [C.c_void_p, C.c_uint64, C.POINTER(C.c_void_p)]),
    "pw_future_retain": (C.c_int, [C.c_void_p, C.c_uint64]),
    "pw_future_release": (C.c_int, [C.c_void_p, C.c_uint64]),
    "pw_model_create": (C.c_int, [C.c_void_p, C.POINTER(LMConfigC), C.POINTER(C.c_void_p)]),
    "pw_model_destroy": (C.c_int, [C.c_void_p]),
    "pw_model_param_count": (C.c_int64, [C.c_void_p]),
    "pw_model_param_info": (C.c_int, [C.c_void_p, C.c_int64, C.c_char_p, C.c_int, C.POINTER(C.c_int64)]),
    "pw_model_import": (C.c_int, [C.c_void_p, C.c_int, C.c_int64, C.c_void_p, C.c_int]),
    "pw_model_export": (C.c_int, [C.c_void_p, C.c_int, C.c_int64, C.c_void_p]),
    "pw_model_zero_grads": (C.c_int, [C.c_void_p]),
    "pw_model_apply_optimizer": (C.c_int, [C.c_void_p]),
    "pw_model_export_activation": (C.c_int, [C.c_void_p, C.c_char_p, C.c_int, C.c_void_p, C.c_int64]),
    "pw_model_step_flops": (C.c_double, [C.POINTER(LMConfigC)]),
    "pw_encdec_create": (C.c_int, [C.c_void_p, C.POINTER(EncDecConfigC), C.POINTER(C.c_void_p)]),
    "pw_encdec_destroy": (C.c_int, [C.c_void_p]),
    "pw_encdec_param_count": (C.c_int64, [C.c_void_p]),
    "pw_encdec_param_info": (C.c_int, [C.c_void_p, C.c_int64, C.c_char_p, C.c_int, C.POINTER(C.c_int64)]),
    "pw_encdec_import": (C.c_int, [C.c_void_p, C.c_int, C.c_int64, C.c_void_p, C.c_int]),
    "pw_encdec_export": (C.c_int, [C.c_void_p, C.c_int, C.c_int64, C.c_void_p]),
    "pw_encdec_export_activation": (C.c_int, [C.c_void_p, C.c_char_p, C.c_void_p, C.c_int64]),
    "pw_encdec_step_flops": (C.c_double, [C.POINTER(EncDecConfigC)]),
    "pw_profile_begin": (C.c_int, [C.c_void_p]),
    "pw_profile_pause": (C.c_int, [C.c_void_p]),
    "pw_profile_end": (C.c_int, [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "pw_profile_fused_update": (C.c_int, [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "pw_profile_gemm_shapes": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(C.c_int32)]),
    "pw_op_gemm": (C.c_int, [C.c_void_p, C.POINTER(GemmArgs)]),
    "pw_op_gemm_pair": (C.c_int, [C.c_void_p, C.POINTER(GemmArgs), C.POINTER(GemmArgs)]),
    "pw_op_gemm_group": (C.c_int, [C.c_void_p, C.POINTER(GemmArgs), C.c_int]),
    "pw_op_embedding_fwd": (C.c_int, [C.c_void_p] + [C.c_void_p] * 4 + [C.c_int] * 4),
    "pw_op_embedding_bwd": (C.c_int, [C.c_void_p] + [C.c_void_p] * 4 + [C.c_int] * 4),
    "pw_op_layernorm_fwd": (C.c_int, [C.c_void_p, C.c_int] + [C.c_void_p] * 6 + [C.c_int] * 2),
    "pw_op_layernorm_bwd": (C.c_int, [C.c_void_p, C.c_int] + [C.c_void_p] * 12 + [C.c_int] * 3),
    "pw_layernorm_bwd_ws_floats": (C.c_int64, [C.c_int, C.c_int]),
    "pw_op_layernorm_bwd_noalloc": (C.c_int, [C.c_void_p, C.c_int] + [C.c_void_p] * 11 + [C.c_int] * 3),
    "pw_op_attention_fwd": (C.c_int, [C.c_void_p, C.c_int] + [C.c_void_p] * 3 + [C.c_int] * 4),
    "pw_op_attention_bwd": (C.c_int, [C.c_void_p, C.c_int] + [C.c_void_p] * 6 + [C.c_int] * 4),
    "pw_op_mha_fwd": (C.c_int, [C.c_void_p] * 5),
    "pw_op_mha_bwd": (C.c_int, [C.c_void_p] * 8 + [C.c_int64, C.c_void_p, C.c_void_p, C.c_int64]),
    "pw_op_softmax_xent": (C.c_int, [C.c_void_p, C.c_int] + [C.c_void_p] * 4 + [C.c_int] * 3),
    "pw_op_xent_from_stats": (C.c_int, [C.c_void_p] * 6 + [C.c_int] * 2),
    "pw_op_colsum": (C.c_int, [C.c_void_p, C.c_int] + [C.c_void_p] * 3 + [C.c_int64] * 2 + [C.c_int]),
    "pw_colsum_ws_floats": (C.c_int64, [C.c_int64, C.c_int64]),
    "pw_op_sgd": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_float]),
    "pw_op_adam": (C.c_int, [C.c_void_p] + [C.c_void_p] * 5 + [C.c_int64] + [C.c_float] * 4 + [C.c_int]),
}
DECLARED_SYMBOLS = sorted(_SIGS)


def lib():
    """Load libpw.so.  Raises if it has not been built: the product path has no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2203_12533_amd.build`")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(l, name)          # AttributeError if the library lacks a declared symbol
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def make_spec(dtype: int, shape) -> TensorSpec:
    s = TensorSpec()
    s.dtype, s.rank = dtype, len(shape)
    for i, v in enumerate(shape):
        s.dims[i] = int(v)
    return s


_NP_DTYPES = {PW_F32: np.float32, PW_I32: np.int32, PW_BF16: np.uint16}


class Context:
    """pw_ctx: one GPU, one FIFO executor stream."""

    def __init__(self, device: int = 0, stream_ptr: int | None = None):
        self._h = C.c_void_p()
        st = lib().pw_ctx_create(device, C.c_void_p(stream_ptr) if stream_ptr else None, C.byref(self._h))
        if st != PW_OK:
            self._h = None
            raise PwError(st, "pw_ctx_create failed (is a gfx950 GPU visible?)")
        self._models = []

    # -- plumbing
    def _check(self, st: int):
        if st != PW_OK:
            raise PwError(st, lib().pw_last_error(self._h).decode())

    @property
    def handle(self):
        return self._h

    def close(self):
        if self._h is not None:
            for m in list(self._models):
                m.close()
            lib().pw_ctx_destroy(self._h)
            self._h = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def synchronize(self):
        self._check(lib().pw_ctx_synchronize(self._h))

    def stream_ptr(self) -> int:
        return lib().pw_ctx_stream(self._h)

    def set_gate_timeout_ms(self, ms: int):
        self._check(lib().pw_ctx_set_gate_timeout_ms(self._h, ms))

    def stats(self):
        a, b = C.c_int64(), C.c_int64()
        self._check(lib().pw_ctx_stats(self._h, C.byref(a), C.byref(b)))
        return a.value, b.value

    # -- compiled functions
    def compile_fn(self, kind: int, in_specs, out_specs, params: bytes = b"") -> int:
        d = FnDesc()
        d.kind, d.n_in, d.n_out = kind, len(in_specs), len(out_specs)
        for i, s in enumerate(in_specs):
            d.in_[i] = s
        for i, s in enumerate(out_specs):
            d.out[i] = s
        buf = C.create_string_buffer(params, len(params)) if params else None
        d.params = C.cast(buf, C.c_void_p) if buf is not None else None
        d.params_bytes = len(params)
        h = C.c_uint64()
        self._check(lib().pw_compile_fn(self._h, C.byref(d), C.byref(h)))
        return h.value

    def compile_scalar_fn(self, kind: int, n: int, c: float, busy_us: float | None = None,
                          reps: int | None = None) -> int:
        spec = make_spec(PW_F32, (n,))
        vals = [c] if busy_us is None else [c, busy_us] if reps is None else [c, busy_us, reps]
        return self.compile_fn(kind, [spec], [spec], np.asarray(vals, np.float32).tobytes())

    def fn_release(self, fn: int):
        self._check(lib().pw_fn_release(self._h, fn))

    def run_fn(self, fn: int, inputs, n_out: int = 1):
        a_in = (C.c_uint64 * max(1, len(inputs)))(*inputs)
        a_out = (C.c_uint64 * max(1, n_out))()
        self._check(lib().pw_run_fn(self._h, fn, a_in, len(inputs), a_out, n_out))
        return list(a_out[:n_out])

    def chain(self, fns, inputs, n_out: int = 1, mode: int = PW_STREAM):
        a_f = (C.c_uint64 * len(fns))(*fns)
        a_in = (C.c_uint64 * max(1, len(inputs)))(*inputs)
        a_out = (C.c_uint64 * max(1, n_out))()
        self._check(lib().pw_chain(self._h, a_f, len(fns), a_in, len(inputs), a_out, n_out, mode))
        return list(a_out[:n_out])

    def set_owner(self, owner: int):
        self._check(lib().pw_ctx_set_owner(self._h, owner))

    def owner_collect(self, owner: int) -> int:
        n = C.c_int64()
        self._check(lib().pw_owner_collect(self._h, owner, C.byref(n)))
        return n.value

    def set_memory_limit(self, nbytes: int):
        self._check(lib().pw_ctx_set_memory_limit(self._h, nbytes))

    def set_executors(self, n: int):
        self._check(lib().pw_ctx_set_executors(self._h, n))

    def set_executor_prep_us(self, us: int):
        self._check(lib().pw_ctx_set_executor_prep_us(self._h, us))

    def pipeline(self, fns, executor_of, f_in: int, dispatch: int = PW_DISPATCH_PARALLEL) -> int:
        a_f = (C.c_uint64 * len(fns))(*fns)
        a_e = (C.c_int32 * len(fns))(*executor_of)
        out = C.c_uint64()
        self._check(lib().pw_pipeline(self._h, a_f, a_e, len(fns), f_in, C.byref(out), dispatch))
        return out.value

    def train_step(self, step_fn: int, tokens_future: int) -> int:
        out = C.c_uint64()
        self._check(lib().pw_train_step(self._h, step_fn, tokens_future, C.byref(out)))
        return out.value

    # -- futures
    def future_from_host(self, arr: np.ndarray, dtype: int | None = None) -> int:
        arr = np.ascontiguousarray(arr)
        if dtype is None:
            dtype = {np.dtype(np.float32): PW_F32, np.dtype(np.int32): PW_I32, np.dtype(np.uint16): PW_BF16}[arr.dtype]
        spec = make_spec(dtype, arr.shape)
        h = C.c_uint64()
        self._check(lib().pw_future_from_host(self._h, arr.ctypes.data_as(C.c_void_p), C.byref(spec), C.byref(h)))
        return h.value

    def future_wrap_device(self, ptr: int, dtype: int, shape) -> int:
        spec = make_spec(dtype, shape)
        h = C.c_uint64()
        self._check(lib().pw_future_wrap_device(self._h, C.c_void_p(ptr), C.byref(spec), C.byref(h)))
        return h.value

    def future_pending(self, dtype: int, shape) -> int:
        spec = make_spec(dtype, shape)
        h = C.c_uint64()
        self._check(lib().pw_future_pending(self._h, C.byref(spec), C.byref(h)))
        return h.value

    def future_resolve(self, f: int, arr: np.ndarray | None):
        if arr is None:
            self._check(lib().pw_future_resolve(self._h, f, None))
        else:
            arr = np.ascontiguousarray(arr)
            self._check(lib().pw_future_resolve(self._h, f, arr.ctypes.data_as(C.c_void_p)))

    def future_query(self, f: int) -> int:
        return lib().pw_future_query(self._h, f)

    def future_spec(self, f: int):
        s = TensorSpec()
        self._check(lib().pw_future_spec(self._h, f, C.byref(s)))
        return s.dtype, tuple(s.dims[i] for i in range(s.rank))

    def future_device_ptr(self, f: int) -> int:
        p = C.c_void_p()
        self._check(lib().pw_future_device_ptr(self._h, f, C.byref(p)))
        return p.value

    def future_retain(self, f: int):
        self._check(lib().pw_future_retain(self._h, f))

    def future_release(self, f: int):
        self._check(lib().pw_future_release(self._h, f))

    def await_(self, f: int, fetch: bool = True):
        """Block until ready; returns the value as a numpy array (bf16 as raw uint16) when fetch."""
        if not fetch:
            self._check(lib().pw_await(self._h, f, None, 0))
            return None
        dtype, shape = self.future_spec(f)
        out = np.empty(shape, dtype=_NP_DTYPES[dtype])
        self._check(lib().pw_await(self._h, f, out.ctypes.data_as(C.c_void_p), out.nbytes))
        return out

    # -- measurement aid
    def profile_begin(self):
        self._check(lib().pw_profile_begin(self._h))

    def profile_pause(self):
        self._check(lib().pw_profile_pause(self._h))

    def profile_end(self):
        n, ms, fl = C.c_int64(), C.c_double(), C.c_double()
        self._check(lib().pw_profile_end(self._h, C.byref(n), C.byref(ms), C.byref(fl)))
        return n.value, ms.value, fl.value

    def profile_fused_update(self):
        """(launches, ms, flops) of the GEMM launches with the Adam epilogue, as of the last profile_end()."""
        n, ms, fl = C.c_int64(), C.c_double(), C.c_double()
        self._check(lib().pw_profile_fused_update(self._h, C.byref(n), C.byref(ms), C.byref(fl)))
        return n.value, ms.value, fl.value

    def profile_gemm_shapes(self):
        """The launches of the last profile_end() by shape: a list of dicts, largest total time first."""
        n = C.c_int32()
        self._check(lib().pw_profile_gemm_shapes(self._h, None, 0, C.byref(n)))
        rows = (GemmShapeRow * max(n.value, 1))()
        self._check(lib().pw_profile_gemm_shapes(self._h, C.cast(rows, C.c_void_p), n.value, C.byref(n)))
        return [{f: getattr(r, f) for f, _ in GemmShapeRow._fields_} for r in rows[:n.value]]

    # -- model
    def model(self, cfg, fused_update: bool = False, fused_head_loss: bool = False) -> "Model":
        return Model(self, cfg, fused_update, fused_head_loss)

    def encdec(self, cfg, fused_update: bool = False) -> "EncDec":
        return EncDec(self, cfg, fused_update)

    # -- single kernels (device pointers as ints)
    def op(self, name: str, *args):
        self._check(getattr(lib(), "pw_op_" + name)(self._h, *args))

    def gemm(self, **kw):
        a = _gemm_args(kw)
        self._check(lib().pw_op_gemm(self._h, C.byref(a)))

    def mha_fwd(self, args: "MhaArgs", o: int, lse: int, o_lo: int = 0):
        self._check(lib().pw_op_mha_fwd(self._h, C.byref(args), o, o_lo or None, lse))

    def mha_bwd(self, args: "MhaArgs", o: int, dout: int, lse: int, delta: int, dq: int, lddq: int, dk: int, dv: int,
                lddkv: int, o_lo: int = 0):
        self._check(lib().pw_op_mha_bwd(self._h, C.byref(args), o, o_lo or None, dout, lse, delta, dq, lddq, dk, dv, lddkv))

    def gemm_group(self, kws: list):
        arr = (GemmArgs * len(kws))()
        keep = []
        for a, kw in zip(arr, kws):
            keep.append(_gemm_args(kw, a))
        self._check(lib().pw_op_gemm_group(self._h, arr, len(kws)))

    def gemm_pair(self, kw0: dict, kw1: dict):
        a0, a1 = _gemm_args(kw0), _gemm_args(kw1)
        self._check(lib().pw_op_gemm_pair(self._h, C.byref(a0), C.byref(a1)))


def _gemm_args(kw: dict, a: "GemmArgs | None" = None) -> "GemmArgs":
    """Fills a pw_gemm_args from keywords; adam= / xent= take an AdamEpilogue / XentEpilogue, which the returned
    structure keeps alive (ctypes holds the pointee of a pointer field set from a structure)."""
    a = GemmArgs() if a is None else a
    for k, v in kw.items():
        if k in ("adam", "xent"):
            setattr(a, k, C.pointer(v))
        else:
            setattr(a, k, v)
    return a


class Node(C.Structure):
    _fields_ = [("fn", C.c_uint64), ("n_in", C.c_int32), ("inputs", C.c_int32 * 8)]


class Program:
    """pw_program: a traced DAG of compiled functions.  Values: inputs 0..n_inputs-1, then node outputs in order."""

    def __init__(self, ctx: Context, input_specs, nodes, outputs):
        """nodes: list of (fn handle, [value ids]); outputs: value ids."""
        self._ctx = ctx
        specs = (TensorSpec * max(1, len(input_specs)))(*input_specs)
        arr = (Node * len(nodes))()
        for k, (fn, ins) in enumerate(nodes):
            arr[k].fn = fn
            arr[k].n_in = len(ins)
            for j, v in enumerate(ins):
                arr[k].inputs[j] = v
        outs = (C.c_int32 * len(outputs))(*outputs)
        self._n_out = len(outputs)
        self._h = C.c_void_p()
        ctx._check(lib().pw_program_create(ctx.handle, specs, len(input_specs), arr, len(nodes), outs, len(outputs),
                                           C.byref(self._h)))

    def run(self, inputs, mode: int = PW_STREAM):
        a_in = (C.c_uint64 * max(1, len(inputs)))(*inputs)
        a_out = (C.c_uint64 * self._n_out)()
        self._ctx._check(lib().pw_program_run(self._ctx.handle, self._h, a_in, len(inputs), a_out, self._n_out, mode))
        return list(a_out)

    def close(self):
        if self._h:
            lib().pw_program_destroy(self._h)
            self._h = None


class SchedSlice(C.Structure):
    _fields_ = [("client", C.c_int32), ("computations", C.c_int32), ("start_ms", C.c_float), ("end_ms", C.c_float)]


class Scheduler:
    """pw_sched: several clients, one executor.  submit / wait / stats may be called from any thread."""

    def __init__(self, ctx: Context, policy: int = PW_SCHED_FIFO, max_in_flight: int = 4):
        self._ctx = ctx
        self._h = C.c_void_p()
        ctx._check(lib().pw_sched_create(ctx.handle, policy, max_in_flight, C.byref(self._h)))

    def _check(self, st: int):
        if st != PW_OK:
            raise PwError(st, lib().pw_last_error(self._ctx.handle).decode())

    def add_client(self, weight: float = 1.0) -> int:
        cid = C.c_int()
        self._check(lib().pw_sched_add_client(self._h, weight, C.byref(cid)))
        return cid.value

    def submit(self, client: int, fns, f_in: int) -> int:
        a_f = (C.c_uint64 * len(fns))(*fns)
        t = C.c_uint64()
        self._check(lib().pw_sched_submit(self._h, client, a_f, len(fns), f_in, C.byref(t)))
        return t.value

    def wait(self, ticket: int, n_floats: int = 0):
        out = np.empty(n_floats, np.float32)
        self._check(lib().pw_sched_wait(self._h, ticket, out.ctypes.data_as(C.c_void_p) if n_floats else None, n_floats * 4))
        return out

    def client_fail(self, client: int) -> int:
        n = C.c_int64()
        self._check(lib().pw_sched_client_fail(self._h, client, C.byref(n)))
        return n.value

    def stalls(self):
        n, ms = C.c_int64(), C.c_double()
        self._check(lib().pw_sched_stalls(self._h, C.byref(n), C.byref(ms)))
        return n.value, ms.value

    def drain(self):
        self._check(lib().pw_sched_drain(self._h))

    def client_stats(self, client: int):
        p, n, ms = C.c_int64(), C.c_int64(), C.c_double()
        self._check(lib().pw_sched_client_stats(self._h, client, C.byref(p), C.byref(n), C.byref(ms)))
        return p.value, n.value, ms.value

    def trace(self):
        n = C.c_int()
        self._check(lib().pw_sched_trace(self._h, None, 0, C.byref(n)))
        arr = (SchedSlice * max(1, n.value))()
        self._check(lib().pw_sched_trace(self._h, arr, n.value, C.byref(n)))
        return [(a.client, a.computations, a.start_ms, a.end_ms) for a in arr[:n.value]]

    def close(self):
        if self._h:
            lib().pw_sched_destroy(self._h)
            self._h = None


def lm_config_c(cfg, fused_update: bool = False, fused_head_loss: bool = False) -> LMConfigC:
    """From the generator module's LMConfig (or any object with the same fields); the two fusion switches are
    choices of the GPU path, not part of the workload."""
    return LMConfigC(cfg.n_layer, cfg.d_model, cfg.n_head, cfg.d_ff, cfg.vocab, cfg.seq, cfg.batch, int(cfg.bf16),
                     {"sgd": 1, "adam": 2}[cfg.optimizer], cfg.lr, cfg.beta1, cfg.beta2, cfg.eps,
                     int(cfg.has_embed), int(cfg.has_head), cfg.n_microbatch, int(fused_update), int(fused_head_loss))


def step_flops(cfg) -> float:
    c = lm_config_c(cfg)
    return lib().pw_model_step_flops(C.byref(c))


def encdec_config_c(cfg, fused_update: bool = False) -> EncDecConfigC:
    """From the generator module's EncDecConfig (or any object with the same fields)."""
    return EncDecConfigC(cfg.n_enc_layer, cfg.n_dec_layer, cfg.d_model, cfg.n_head, cfg.d_ff, cfg.vocab, cfg.src_len,
                         cfg.tgt_len, cfg.batch, int(cfg.bf16), {"sgd": 1, "adam": 2}[cfg.optimizer], cfg.lr, cfg.beta1,
                         cfg.beta2, cfg.eps, int(fused_update))


def encdec_step_flops(cfg) -> float:
    c = encdec_config_c(cfg)
    return lib().pw_encdec_step_flops(C.byref(c))


class _ParamModel:
    """What pw_model and pw_encdec have in common: named fp32 parameter tensors with gradients and optimiser state
    that can be imported and exported one tensor at a time.  `_prefix` names the C entry points."""
    _prefix = ""

    def _fn(self, name: str):
        return getattr(lib(), f"{self._prefix}_{name}")

    def _read_param_table(self):
        self.names, self.numel = [], {}
        name = C.create_string_buffer(64)
        n = C.c_int64()
        for i in range(self._fn("param_count")(self._h)):
            self._fn("param_info")(self._h, i, name, 64, C.byref(n))
            self.names.append(name.value.decode())
            self.numel[self.names[-1]] = n.value
        self._index = {k: i for i, k in enumerate(self.names)}

    def close(self):
        if self._h is not None:
            self._fn("destroy")(self._h)
            self._h = None
            if self in self.ctx._models:
                self.ctx._models.remove(self)

    def import_(self, part: int, name: str, arr: np.ndarray):
        arr = np.ascontiguousarray(arr, dtype=np.float32)
        assert arr.size == self.numel[name], (name, arr.size, self.numel[name])
        self.ctx._check(self._fn("import")(self._h, part, self._index[name], arr.ctypes.data_as(C.c_void_p), 0))

    def import_device(self, part: int, name: str, ptr: int):
        self.ctx._check(self._fn("import")(self._h, part, self._index[name], C.c_void_p(ptr), 1))

    def load_params(self, params: dict):
        for k in self.names:
            self.import_(PW_PARAMS, k, params[k])

    def export(self, part: int, name: str, shape=None) -> np.ndarray:
        out = np.empty(self.numel[name], dtype=np.float32)
        self.ctx._check(self._fn("export")(self._h, part, self._index[name], out.ctypes.data_as(C.c_void_p)))
        return out.reshape(shape) if shape is not None else out

    def export_all(self, part: int, like: dict) -> dict:
        return {k: self.export(part, k, like[k].shape) for k in self.names}


class EncDec(_ParamModel):
    """pw_encdec: parameters, optimiser state and the static activation plan of one encoder-decoder model."""
    _prefix = "pw_encdec"

    def __init__(self, ctx: "Context", cfg, fused_update: bool = False):
        self.ctx, self.cfg = ctx, cfg
        self._h = C.c_void_p()
        c = encdec_config_c(cfg, fused_update)
        ctx._check(lib().pw_encdec_create(ctx.handle, C.byref(c), C.byref(self._h)))
        ctx._models.append(self)
        self._read_param_table()

    def export_activation(self, name: str, numel: int) -> np.ndarray:
        out = np.empty(numel, dtype=np.float32)
        self.ctx._check(lib().pw_encdec_export_activation(self._h, name.encode(), out.ctypes.data_as(C.c_void_p), numel))
        return out

    def compile_train_step(self) -> int:
        cfg = self.cfg
        params = C.c_void_p(self._h.value)
        return self.ctx.compile_fn(PW_FN_ENCDEC_TRAIN_STEP,
                                   [make_spec(PW_I32, (cfg.batch, cfg.src_len)), make_spec(PW_I32, (cfg.batch, cfg.tgt_len + 1))],
                                   [make_spec(PW_F32, (1,))], bytes(params))


class Model(_ParamModel):
    """pw_model: parameters, optimiser state and the static activation plan of one LM (or pipeline stage)."""
    _prefix = "pw_model"

    def __init__(self, ctx: Context, cfg, fused_update: bool = False, fused_head_loss: bool = False):
        self.ctx, self.cfg = ctx, cfg
        self._h = C.c_void_p()
        c = lm_config_c(cfg, fused_update, fused_head_loss)
        ctx._check(lib().pw_model_create(ctx.handle, C.byref(c), C.byref(self._h)))
        ctx._models.append(self)
        self._read_param_table()

    def export_activation(self, name: str, numel: int, microbatch: int = 0) -> np.ndarray:
        out = np.empty(numel, dtype=np.float32)
        self.ctx._check(lib().pw_model_export_activation(self._h, name.encode(), microbatch,
                                                         out.ctypes.data_as(C.c_void_p), numel))
        return out

    def zero_grads(self):
        self.ctx._check(lib().pw_model_zero_grads(self._h))

    def apply_optimizer(self):
        self.ctx._check(lib().pw_model_apply_optimizer(self._h))

    def compile_train_step(self) -> int:
        cfg = self.cfg
        params = C.c_void_p(self._h.value)
        return self.ctx.compile_fn(PW_FN_LM_TRAIN_STEP, [make_spec(PW_I32, (cfg.batch, cfg.seq + 1))],
                                   [make_spec(PW_F32, (1,))], bytes(params))

    def compile_stage(self, kind: int, microbatch: int) -> int:
        cfg = self.cfg
        sp = StageParams(self._h.value, microbatch)
        spec = make_spec(PW_F32, (cfg.batch * cfg.seq, cfg.d_model))
        return self.ctx.compile_fn(kind, [spec], [spec], bytes(sp))
