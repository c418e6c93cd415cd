"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the header
declares, and rejects invalid calls with the documented error codes before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2409_15241_amd import domino, synth

LIB_OK = os.path.exists(domino.LIB_PATH)
pytestmark = pytest.mark.skipif(not LIB_OK, reason="libdomino.so not built (python -m paper_2409_15241_amd.build)")


def header_functions(repo_root):
    text = open(os.path.join(repo_root, "include", "domino.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(domino_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(repo_root):
    lib = domino.load()
    names = header_functions(repo_root)
    assert len(names) >= 20
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(domino.EXPORTS) == names
    assert "gfx950" in domino.domino_version()


def test_binding_exposes_the_same_names():
    for n in domino.EXPORTS:
        assert callable(getattr(domino, n)), n


def cfg(**kw):
    return domino.make_cfg(synth.WORKLOADS["tiny"], **kw)


@pytest.mark.parametrize("kw,code", [
    (dict(p=3), domino.ERR_INDIVISIBLE),             # batch 2 % 3
    (dict(q=3), domino.ERR_INDIVISIBLE),             # hidden 256 % 3
    (dict(tp=3), domino.ERR_INDIVISIBLE),            # heads 4 % 3
    (dict(ffn=1001), domino.ERR_INDIVISIBLE),        # ffn % tp
    (dict(heads=3), domino.ERR_INDIVISIBLE),         # hidden % heads
    (dict(wgrad_per_slice=2), domino.ERR_INVALID_ARG),   # a switch: 0 or 1
    (dict(rank=2), domino.ERR_INVALID_ARG),
    (dict(rank=-1), domino.ERR_INVALID_ARG),
    (dict(batch=0), domino.ERR_INVALID_ARG),
    (dict(arch=7), domino.ERR_INVALID_ARG),
    (dict(norm_eps=0.0), domino.ERR_INVALID_ARG),
    (dict(heads=8, tp=2), domino.ERR_UNSUPPORTED),   # head_dim 32
    (dict(hidden=16384, heads=128), domino.ERR_UNSUPPORTED),
    (dict(q=64), domino.ERR_UNSUPPORTED),            # hidden/q = 4 columns
    (dict(batch=1 << 14, seq=1 << 14, p=1), domino.ERR_UNSUPPORTED),   # tensors beyond 2 GiB
])
def test_invalid_configs_are_rejected(kw, code):
    c = cfg(**kw)
    assert domino.domino_validate_cfg(c) == code
    assert domino.domino_last_error() != ""
    assert domino.domino_saved_bytes(c) == 0 and domino.domino_workspace_bytes(c) == 0


def test_every_workload_validates_and_sizes_are_consistent():
    for sc in synth.WORKLOADS.values():
        c = domino.make_cfg(sc)
        assert domino.domino_validate_cfg(c) == domino.OK, sc.name
        total = domino.domino_saved_bytes(c)
        M = sc.tokens
        want = {"ln1": M * sc.hidden * 2, "qkv": M * 3 * sc.h_local * 2, "ctx": M * sc.h_local * 2,
                "lse": sc.batch * sc.local_heads * sc.seq * 4, "x1": M * sc.hidden * 2, "ln2": M * sc.hidden * 2,
                "pre": M * sc.up_cols * 2, "act": M * sc.f_local * 2, "mean1": M * 4, "rstd2": M * 4}
        spans = []
        for name, size in want.items():
            off, got = domino.domino_saved_slot(c, name)
            assert got == size and off % 256 == 0 and off + got <= total, (sc.name, name)
            spans.append((off, off + got))
        spans.sort()
        assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))
        assert domino.domino_workspace_bytes(c) > 0
    with pytest.raises(domino.DominoError):
        domino.domino_saved_slot(domino.make_cfg(synth.WORKLOADS["tiny"]), "nope")


def _call_fwd(c, params_ptrs, x=1, ap=1, mp=1, saved=1, ws=1, ws_bytes=1 << 40, streams=None, n=1):
    lib = domino.load()
    ps = domino.domino_params(**params_ptrs)
    arr = (C.c_void_p * 1)(None) if streams is None else streams
    return lib.domino_layer_fwd(C.byref(c), C.byref(ps), x, None, None, ap, mp, None, saved, ws, ws_bytes, arr, n)


def test_layer_calls_validate_before_touching_the_gpu():
    """Dummy non-null pointers are never dereferenced: each call must fail in validation."""
    c = cfg()
    full = {n: 0x1000 for n in domino.PARAM_NAMES}
    assert _call_fwd(c, {**full, "w_qkv": None}) == domino.ERR_NULL_POINTER
    assert _call_fwd(c, {**full, "b_up": None}) == domino.ERR_NULL_POINTER        # GPT needs its biases
    assert _call_fwd(c, full, x=None) == domino.ERR_NULL_POINTER
    assert _call_fwd(c, full, ws_bytes=16) == domino.ERR_WORKSPACE_TOO_SMALL
    assert "needed" in domino.domino_last_error()
    assert _call_fwd(c, full, n=0) == domino.ERR_INVALID_ARG
    assert _call_fwd(cfg(p=3), full) == domino.ERR_INDIVISIBLE
    lc = domino.make_cfg(synth.WORKLOADS["tiny-llama"])
    assert _call_fwd(lc, full) == domino.ERR_INVALID_ARG                           # Llama: biases must be NULL
    lib = domino.load()
    ps = domino.domino_params(**full)
    gs = domino.domino_grads(**full)
    arr = (C.c_void_p * 1)(None)
    rc = lib.domino_layer_bwd(C.byref(c), C.byref(ps), 1, 1, None, None, None, 1, 1, 1, C.byref(gs), 0, 1, 1 << 40, arr, 1)
    assert rc == domino.ERR_NULL_POINTER                                           # dy missing
    gs2 = domino.domino_grads(**{**full, "w_o": None})
    rc = lib.domino_layer_bwd(C.byref(c), C.byref(ps), 1, 1, 1, None, None, 1, 1, 1, C.byref(gs2), 0, 1, 1 << 40, arr, 1)
    assert rc == domino.ERR_NULL_POINTER
    # dx must not overlap dy: a weight gradient may read dy after dx has been written
    rc = lib.domino_layer_bwd(C.byref(c), C.byref(ps), 1, 1, 0x100000, None, None, 1, 1, 0x100100, C.byref(gs), 0, 1, 1 << 40, arr, 1)
    assert rc == domino.ERR_INVALID_ARG and "overlaps" in domino.domino_last_error()


def test_single_kernel_entry_points_validate():
    lib = domino.load()
    g = lambda **kw: lib.domino_gemm(kw.get("layout", 0), kw.get("epi", 0), kw.get("tile", -1), 1, kw.get("lda", 64), 1, 64,
                                     kw.get("C", 1), 64, kw.get("M", 64), 64, kw.get("K", 64), None, kw.get("aux"), 64, 0, 0, 1, None)
    assert g(C=None) == domino.ERR_NULL_POINTER
    assert g(M=60) == domino.ERR_UNSUPPORTED
    assert g(K=0) == domino.ERR_INVALID_ARG
    assert g(layout=0, epi=domino.EPI_ACC_F32) == domino.ERR_INVALID_ARG
    assert g(layout=2, epi=domino.EPI_STORE) == domino.ERR_INVALID_ARG
    assert g(epi=domino.EPI_BIAS_GELU) == domino.ERR_NULL_POINTER                 # aux missing
    assert g(tile=5) == domino.ERR_INVALID_ARG
    assert lib.domino_attention_fwd(1, 192, 1, 16, 1, 48, 1, 1, None) == domino.ERR_UNSUPPORTED
    assert lib.domino_attention_fwd(1, 100, 1, 16, 1, 64, 1, 1, None) == domino.ERR_INVALID_ARG
    assert lib.domino_norm_fwd(1, None, None, None, 1, None, None, 1, None, 1, 4, 12, 0, 1e-5, None) == domino.ERR_UNSUPPORTED
    assert lib.domino_norm_fwd(None, None, None, None, 1, None, None, 1, None, 1, 4, 16, 0, 1e-5, None) == domino.ERR_NULL_POINTER
    assert lib.domino_rope(1, 64, 4, 4, 0, 2, 1, 64, 10000.0, 0, None) == domino.ERR_INVALID_ARG   # blocks exceed ld
    assert lib.domino_colsum(1, 64, 4, 60, 1, 0, 1, None) == domino.ERR_UNSUPPORTED
    assert lib.domino_norm_bwd_scratch_floats(2048, 5120) == 2 * 128 * 5120
    assert lib.domino_profile_classes() >= 18 and lib.domino_profile_name(1) == b"gemm_qkv"
    assert lib.domino_profile_read(99, None, None) == domino.ERR_INVALID_ARG
    assert lib.domino_profile_records() == 0
    assert lib.domino_profile_record(0, None, None, None, None) == domino.ERR_NULL_POINTER


def test_capture_is_offered_for_the_pools_that_replay_bit_for_bit_only():
    """Pools of 1, 2 or 4 streams of which 1, 2 or 4 carry slices; everything else is refused (3 and 8 have aborted)."""
    ok = {(n, p) for n in range(1, 10) for p in range(1, 10) if domino.domino_capture_supported(n, p)}
    want = {(n, p) for n in (1, 2, 4) for p in range(1, 10) if min(n, p) in (1, 2, 4)}
    assert ok == want
    assert not domino.domino_capture_supported(3, 4) and not domino.domino_capture_supported(8, 4)
    assert not domino.domino_capture_supported(0, 4) and not domino.domino_capture_supported(4, 0)


def test_no_warning_before_any_layer_call_and_probe_validates():
    lib = domino.load()
    assert domino.domino_last_warning() == ""
    assert lib.domino_mfma_probe(None, 1, 1, 1, 1, None, None) == domino.ERR_NULL_POINTER
    assert lib.domino_mfma_probe(1, 1, 1, 0, 1, None, None) == domino.ERR_INVALID_ARG
    assert lib.domino_mfma_probe(1, 1, 1, 1, 0, None, None) == domino.ERR_INVALID_ARG


def test_tuner_candidates_cut_exactly():
    from paper_2409_15241_amd import synth, tune
    sc = synth.WORKLOADS["gpt3-13b"]
    pairs = tune.candidates(sc)
    assert (4, 2) in pairs and (1, 1) in pairs
    assert all(sc.batch % p == 0 and sc.hidden % q == 0 for p, q in pairs)
    assert (8, 1) not in pairs          # batch 4 cannot be cut into 8 row slices
