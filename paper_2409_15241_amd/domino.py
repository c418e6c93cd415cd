"""ctypes binding of libdomino.so: same names as include/domino.h, argument marshalling only.

Every function takes torch tensors (device memory; their ``data_ptr()`` is passed on), ``None`` for
optional pointers, torch streams (their ``cuda_stream`` handle is passed on) and plain numbers.
Nothing is computed here: every step of the path runs in the library's kernels.  There is no
fallback: a missing library raises at load time and a failing call raises ``DominoError``.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdomino.so")

OK = 0
ERR_INVALID_ARG, ERR_INDIVISIBLE, ERR_NULL_POINTER = -1, -2, -3
ERR_WORKSPACE_TOO_SMALL, ERR_UNSUPPORTED, ERR_HIP = -4, -5, -6
ARCH_GPT, ARCH_LLAMA = 0, 1
GEMM_NN, GEMM_NT, GEMM_TN = 0, 1, 2
EPI_STORE, EPI_BIAS_GELU, EPI_SWIGLU, EPI_DGELU, EPI_DSWIGLU, EPI_ACC_F32 = range(6)
FWD_ATTN, FWD_MLP, FWD_ALL = 1, 2, 3
BWD_MLP, BWD_ATTN, BWD_NORM1, BWD_ALL = 1, 2, 4, 7

PARAM_NAMES = ("norm1_g", "norm1_b", "w_qkv", "b_qkv", "w_o", "b_o",
               "norm2_g", "norm2_b", "w_up", "b_up", "w_down", "b_down")
EXPORTS = (
    "domino_validate_cfg", "domino_saved_bytes", "domino_workspace_bytes", "domino_saved_slot",
    "domino_layer_fwd", "domino_layer_bwd", "domino_layer_fwd_parts", "domino_layer_bwd_parts",
    "domino_stack_workspace_bytes", "domino_stack_fwd", "domino_stack_bwd",
    "domino_gemm", "domino_gemm_rope", "domino_attention_bwd_rope", "domino_norm_fwd",
    "domino_norm_bwd_scratch_floats", "domino_norm_bwd", "domino_attention_fwd", "domino_attention_bwd",
    "domino_rope", "domino_colsum", "domino_colsum_noalloc", "domino_mfma_probe", "domino_profile_enable", "domino_profile_classes",
    "domino_profile_name", "domino_profile_read", "domino_profile_reset", "domino_profile_records",
    "domino_profile_record", "domino_last_error", "domino_last_warning", "domino_capture_supported",
    "domino_version", "domino_shutdown",
)


class DominoError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"domino error {code}: {text}")
        self.code = code


class domino_cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("hidden", "heads", "tp", "rank", "p", "q", "batch", "seq", "ffn",
                                         "arch", "gelu_tanh")] + [("norm_eps", C.c_float), ("rope_base", C.c_float),
                                                                  ("wgrad_per_slice", C.c_int32)]


class domino_params(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in PARAM_NAMES]


class domino_grads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in PARAM_NAMES]


STACK_FWD_FIELDS = ("attn_others", "mlp_others", "attn_partial", "mlp_partial", "y", "saved")
STACK_BWD_FIELDS = ("x", "saved", "dln2_others", "dln1_others", "dln2_partial", "dln1_partial")


class domino_stack_fwd_io(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in STACK_FWD_FIELDS]


class domino_stack_bwd_io(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in STACK_BWD_FIELDS]


_lib: Optional[C.CDLL] = None


def load() -> C.CDLL:
    """Load the library (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2409_15241_amd.build`")
    # The caller's device memory and streams come from torch, which ships its own HIP runtime under
    # the same soname: load torch first so that the library binds to that one runtime instead of
    # bringing a second copy into the process (handles from one are invalid in the other).
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, f32, sz = C.c_void_p, C.c_int, C.c_int64, C.c_float, C.c_size_t
    cfgp = C.POINTER(domino_cfg)
    sig = {
        "domino_validate_cfg": (i32, [cfgp]),
        "domino_saved_bytes": (sz, [cfgp]),
        "domino_workspace_bytes": (sz, [cfgp]),
        "domino_saved_slot": (i32, [cfgp, C.c_char_p, C.POINTER(sz), C.POINTER(sz)]),
        "domino_layer_fwd": (i32, [cfgp, C.POINTER(domino_params), vp, vp, vp, vp, vp, vp, vp, vp, sz,
                                   C.POINTER(vp), i32]),
        "domino_layer_bwd": (i32, [cfgp, C.POINTER(domino_params), vp, vp, vp, vp, vp, vp, vp, vp,
                                   C.POINTER(domino_grads), i32, vp, sz, C.POINTER(vp), i32]),
        "domino_layer_fwd_parts": (i32, [cfgp, C.POINTER(domino_params), vp, vp, vp, vp, vp, vp, vp, vp, sz,
                                         C.POINTER(vp), i32, i32]),
        "domino_layer_bwd_parts": (i32, [cfgp, C.POINTER(domino_params), vp, vp, vp, vp, vp, vp, vp, vp,
                                         C.POINTER(domino_grads), i32, vp, sz, C.POINTER(vp), i32, i32]),
        "domino_stack_workspace_bytes": (sz, [cfgp, i32]),
        "domino_stack_fwd": (i32, [cfgp, i32, C.POINTER(domino_params), vp, C.POINTER(domino_stack_fwd_io), vp, sz,
                                   C.POINTER(vp), i32]),
        "domino_stack_bwd": (i32, [cfgp, i32, C.POINTER(domino_params), vp, C.POINTER(domino_stack_bwd_io), vp,
                                   C.POINTER(domino_grads), i32, vp, sz, C.POINTER(vp), i32]),
        "domino_gemm": (i32, [i32, i32, i32, vp, i64, vp, i64, vp, i64, i32, i32, i32, vp, vp, i64, i32, i32, i32, vp]),
        "domino_gemm_rope": (i32, [i32, vp, i64, vp, i64, vp, i64, i32, i32, i32, i32, i32, i32, f32, vp]),
        "domino_attention_bwd_rope": (i32, [vp, i64, vp, vp, vp, vp, vp, i32, i32, i32, i32, f32, vp]),
        "domino_norm_fwd": (i32, [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, f32, vp]),
        "domino_norm_bwd_scratch_floats": (sz, [i32, i32]),
        "domino_norm_bwd": (i32, [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, vp]),
        "domino_attention_fwd": (i32, [vp, i64, i32, i32, i32, i32, vp, vp, vp]),
        "domino_attention_bwd": (i32, [vp, i64, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp]),
        "domino_rope": (i32, [vp, i64, i32, i32, i32, i32, i32, i32, f32, i32, vp]),
        "domino_colsum": (i32, [vp, i64, i32, i32, vp, i32, vp, vp]),
        "domino_colsum_noalloc": (i32, [vp, i64, i32, i32, vp, i32, vp]),
        "domino_mfma_probe": (i32, [vp, vp, vp, i32, i32, C.POINTER(C.c_double), vp]),
        "domino_profile_enable": (i32, [i32]),
        "domino_profile_classes": (i32, []),
        "domino_profile_name": (C.c_char_p, [i32]),
        "domino_profile_read": (i32, [i32, C.POINTER(C.c_double), C.POINTER(i32)]),
        "domino_profile_reset": (i32, []),
        "domino_profile_records": (i32, []),
        "domino_profile_record": (i32, [i32, C.POINTER(i32), C.POINTER(C.c_void_p), C.POINTER(C.c_double), C.POINTER(C.c_double)]),
        "domino_last_error": (C.c_char_p, []),
        "domino_last_warning": (C.c_char_p, []),
        "domino_capture_supported": (i32, [i32, i32]),
        "domino_version": (C.c_char_p, []),
        "domino_shutdown": (None, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def _check(rc: int) -> None:
    if rc != OK:
        raise DominoError(rc, load().domino_last_error().decode())


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous() or t.dim() == 2, "tensors must be contiguous (or 2-D row-strided views)"
    return t.data_ptr()


def _stream(s) -> Optional[int]:
    if s is None:
        return None
    return s if isinstance(s, int) else s.cuda_stream


def _streams(streams: Sequence):
    arr = (C.c_void_p * len(streams))(*[_stream(s) for s in streams])
    return arr, len(streams)


def make_cfg(sc=None, **kw) -> domino_cfg:
    """domino_cfg from a synth.ShardConfig-like object and/or keyword overrides."""
    vals = {}
    if sc is not None:
        for n in ("hidden", "heads", "tp", "rank", "p", "q", "batch", "seq", "ffn", "arch", "gelu_tanh",
                  "norm_eps", "rope_base"):
            vals[n] = getattr(sc, n)
        vals["wgrad_per_slice"] = int(getattr(sc, "wgrad_per_slice", 0))
    vals.update(kw)
    vals.setdefault("gelu_tanh", 1)
    vals.setdefault("norm_eps", 1e-5)
    vals.setdefault("rope_base", 10000.0)
    vals.setdefault("arch", ARCH_GPT)
    return domino_cfg(**vals)


def _params_struct(cls, tensors: Dict[str, object]):
    return cls(**{n: _ptr(tensors.get(n)) for n in PARAM_NAMES})


# --------------------------------------------------------------------------- layout queries
def domino_validate_cfg(cfg: domino_cfg) -> int:
    return load().domino_validate_cfg(C.byref(cfg))


def domino_saved_bytes(cfg: domino_cfg) -> int:
    return load().domino_saved_bytes(C.byref(cfg))


def domino_workspace_bytes(cfg: domino_cfg) -> int:
    return load().domino_workspace_bytes(C.byref(cfg))


def domino_saved_slot(cfg: domino_cfg, name: str):
    off, size = C.c_size_t(), C.c_size_t()
    _check(load().domino_saved_slot(C.byref(cfg), name.encode(), C.byref(off), C.byref(size)))
    return off.value, size.value


def domino_last_error() -> str:
    return load().domino_last_error().decode()


def domino_last_warning() -> str:
    return load().domino_last_warning().decode()


def domino_capture_supported(nstreams: int, p: int) -> bool:
    return bool(load().domino_capture_supported(nstreams, p))


def domino_version() -> str:
    return load().domino_version().decode()


def domino_shutdown() -> None:
    load().domino_shutdown()


# --------------------------------------------------------------------------- the layer
def domino_layer_fwd(cfg, params, x, attn_others, mlp_others, attn_partial, mlp_partial, y,
                     saved, workspace, streams) -> None:
    arr, n = _streams(streams)
    ps = _params_struct(domino_params, params)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().domino_layer_fwd(C.byref(cfg), C.byref(ps), _ptr(x), _ptr(attn_others), _ptr(mlp_others),
                                   _ptr(attn_partial), _ptr(mlp_partial), _ptr(y), _ptr(saved), _ptr(workspace),
                                   ws_bytes, arr, n))


def domino_layer_bwd(cfg, params, saved, x, dy, dln2_others, dln1_others, dln2_partial, dln1_partial, dx,
                     grads, accumulate, workspace, streams) -> None:
    arr, n = _streams(streams)
    ps = _params_struct(domino_params, params)
    gs = _params_struct(domino_grads, grads)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().domino_layer_bwd(C.byref(cfg), C.byref(ps), _ptr(saved), _ptr(x), _ptr(dy), _ptr(dln2_others),
                                   _ptr(dln1_others), _ptr(dln2_partial), _ptr(dln1_partial), _ptr(dx),
                                   C.byref(gs), int(accumulate), _ptr(workspace), ws_bytes, arr, n))


def domino_layer_fwd_parts(cfg, params, x, attn_others, mlp_others, attn_partial, mlp_partial, y,
                           saved, workspace, streams, parts) -> None:
    arr, n = _streams(streams)
    ps = _params_struct(domino_params, params)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().domino_layer_fwd_parts(C.byref(cfg), C.byref(ps), _ptr(x), _ptr(attn_others), _ptr(mlp_others),
                                         _ptr(attn_partial), _ptr(mlp_partial), _ptr(y), _ptr(saved),
                                         _ptr(workspace), ws_bytes, arr, n, int(parts)))


def domino_layer_bwd_parts(cfg, params, saved, x, dy, dln2_others, dln1_others, dln2_partial, dln1_partial, dx,
                           grads, accumulate, workspace, streams, parts) -> None:
    arr, n = _streams(streams)
    ps = _params_struct(domino_params, params)
    gs = _params_struct(domino_grads, grads)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().domino_layer_bwd_parts(C.byref(cfg), C.byref(ps), _ptr(saved), _ptr(x), _ptr(dy),
                                         _ptr(dln2_others), _ptr(dln1_others), _ptr(dln2_partial),
                                         _ptr(dln1_partial), _ptr(dx), C.byref(gs), int(accumulate),
                                         _ptr(workspace), ws_bytes, arr, n, int(parts)))


# --------------------------------------------------------------------------- a stack of blocks
def domino_stack_workspace_bytes(cfg: domino_cfg, nlayers: int) -> int:
    return load().domino_stack_workspace_bytes(C.byref(cfg), nlayers)


def _struct_array(cls, fields, dicts):
    return (cls * len(dicts))(*[cls(**{n: _ptr(d.get(n)) for n in fields}) for d in dicts])


def _params_array(cls, dicts):
    return (cls * len(dicts))(*[_params_struct(cls, d) for d in dicts])


def domino_stack_fwd(cfg, params, x, io, workspace, streams) -> None:
    """params: one dict of the twelve tensors per block; io: one dict per block keyed by STACK_FWD_FIELDS."""
    arr, n = _streams(streams)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().domino_stack_fwd(C.byref(cfg), len(params), _params_array(domino_params, params), _ptr(x),
                                   _struct_array(domino_stack_fwd_io, STACK_FWD_FIELDS, io), _ptr(workspace),
                                   ws_bytes, arr, n))


def domino_stack_bwd(cfg, params, dy, io, dx, grads, accumulate, workspace, streams) -> None:
    """io: one dict per block keyed by STACK_BWD_FIELDS; grads: one dict of fp32 tensors per block."""
    arr, n = _streams(streams)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().domino_stack_bwd(C.byref(cfg), len(params), _params_array(domino_params, params), _ptr(dy),
                                   _struct_array(domino_stack_bwd_io, STACK_BWD_FIELDS, io), _ptr(dx),
                                   _params_array(domino_grads, grads), int(accumulate), _ptr(workspace), ws_bytes,
                                   arr, n))


# --------------------------------------------------------------------------- single kernels
def domino_gemm(layout, epilogue, tile, A, lda, B, ldb, Cmat, ldc, M, N, K, bias=None, aux=None, ldaux=0,
                n_split=0, beta=0, gelu_tanh=1, stream=None) -> None:
    _check(load().domino_gemm(layout, epilogue, tile, _ptr(A), lda, _ptr(B), ldb, _ptr(Cmat), ldc, M, N, K,
                              _ptr(bias), _ptr(aux), ldaux, n_split, beta, gelu_tanh, _stream(stream)))


def domino_gemm_rope(tile, A, lda, B, ldb, Cmat, ldc, M, N, K, seq, head_dim, rope_cols, base, stream=None) -> None:
    _check(load().domino_gemm_rope(tile, _ptr(A), lda, _ptr(B), ldb, _ptr(Cmat), ldc, M, N, K, seq, head_dim, rope_cols,
                                   base, _stream(stream)))


def domino_attention_bwd_rope(qkv, ld, ctx, dctx, lse, dqkv, dot, batch, seq, heads, head_dim, base, stream=None) -> None:
    _check(load().domino_attention_bwd_rope(_ptr(qkv), ld, _ptr(ctx), _ptr(dctx), _ptr(lse), _ptr(dqkv), _ptr(dot),
                                            batch, seq, heads, head_dim, base, _stream(stream)))


def domino_norm_fwd(x, add1, add2, vec, gamma, beta, xsum, y, mean, rstd, rows, h, rms, eps, stream=None) -> None:
    _check(load().domino_norm_fwd(_ptr(x), _ptr(add1), _ptr(add2), _ptr(vec), _ptr(gamma), _ptr(beta), _ptr(xsum),
                                  _ptr(y), _ptr(mean), _ptr(rstd), rows, h, int(rms), eps, _stream(stream)))


def domino_norm_bwd_scratch_floats(rows, h) -> int:
    return load().domino_norm_bwd_scratch_floats(rows, h)


def domino_norm_bwd(ga, gb, x, gamma, mean, rstd, dres, dx, dgamma, dbeta, scratch, rows, h, rms, stream=None) -> None:
    _check(load().domino_norm_bwd(_ptr(ga), _ptr(gb), _ptr(x), _ptr(gamma), _ptr(mean), _ptr(rstd), _ptr(dres),
                                  _ptr(dx), _ptr(dgamma), _ptr(dbeta), _ptr(scratch), rows, h, int(rms),
                                  _stream(stream)))


def domino_attention_fwd(qkv, ld, batch, seq, heads, head_dim, ctx, lse, stream=None) -> None:
    _check(load().domino_attention_fwd(_ptr(qkv), ld, batch, seq, heads, head_dim, _ptr(ctx), _ptr(lse),
                                       _stream(stream)))


def domino_attention_bwd(qkv, ld, ctx, dctx, lse, dqkv, dot, batch, seq, heads, head_dim, stream=None) -> None:
    _check(load().domino_attention_bwd(_ptr(qkv), ld, _ptr(ctx), _ptr(dctx), _ptr(lse), _ptr(dqkv), _ptr(dot),
                                       batch, seq, heads, head_dim, _stream(stream)))


def domino_rope(m, ld, rows, seq, col0, nblocks, heads, head_dim, base, inverse, stream=None) -> None:
    _check(load().domino_rope(_ptr(m), ld, rows, seq, col0, nblocks, heads, head_dim, base, int(inverse),
                              _stream(stream)))


def domino_colsum(g, ld, rows, n, out, accumulate, scratch, stream=None) -> None:
    _check(load().domino_colsum(_ptr(g), ld, rows, n, _ptr(out), int(accumulate), _ptr(scratch), _stream(stream)))


def domino_colsum_noalloc(g, ld, rows, n, out, accumulate, stream=None) -> None:
    _check(load().domino_colsum_noalloc(_ptr(g), ld, rows, n, _ptr(out), int(accumulate), _stream(stream)))


def domino_mfma_probe(a, b, out, blocks, iters, stream=None) -> float:
    """Enqueues the probe; returns the flops of the launch."""
    fl = C.c_double()
    _check(load().domino_mfma_probe(_ptr(a), _ptr(b), _ptr(out), blocks, iters, C.byref(fl), _stream(stream)))
    return fl.value


# --------------------------------------------------------------------------- instrumentation
def domino_profile_enable(on: bool) -> None:
    _check(load().domino_profile_enable(int(on)))


def domino_profile_classes() -> int:
    return load().domino_profile_classes()


def domino_profile_name(cls: int) -> str:
    return load().domino_profile_name(cls).decode()


def domino_profile_read(cls: int):
    ms, n = C.c_double(), C.c_int()
    _check(load().domino_profile_read(cls, C.byref(ms), C.byref(n)))
    return ms.value, n.value


def domino_profile_reset() -> None:
    _check(load().domino_profile_reset())


def domino_profile_records() -> int:
    return load().domino_profile_records()


def domino_profile_record(index: int):
    """(step class name, stream handle, start ms, stop ms) of profiled launch `index`, times after record 0's start."""
    cls, st, a, b = C.c_int(), C.c_void_p(), C.c_double(), C.c_double()
    _check(load().domino_profile_record(index, C.byref(cls), C.byref(st), C.byref(a), C.byref(b)))
    return domino_profile_name(cls.value), st.value, a.value, b.value
