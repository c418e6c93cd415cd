"""A stack of blocks through domino_stack_fwd / domino_stack_bwd: parity with the fp64 oracle's composed
blocks, and bitwise identity with one domino_layer_fwd / domino_layer_bwd call per block (same kernels, same
order of every sum; only the waits between streams differ)."""
import numpy as np
import pytest

from oracle import domino_oracle as O
from paper_2409_15241_amd import synth

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

TOL = 2e-2
SAVED_NAMES = ("ln1", "qkv", "ctx", "lse", "x1", "ln2", "pre", "act", "mean1", "rstd1", "mean2", "rstd2")
OUT_KEYS = ("attn_partial", "mlp_partial", "y", "dln2_partial", "dln1_partial")


@pytest.fixture(scope="module")
def H():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2409_15241_amd import domino, harness
    domino.load()
    return harness


def f64(d):
    return {k: (None if v is None else v.astype(np.float64)) for k, v in d.items()}


def relerr(got, ref):
    return float(np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-30))


def run_stack(H, sc, params, others, x, dy, nstreams):
    st = H.StackBuffers(sc, params, x, dy, others, nstreams=nstreams)
    st.forward()
    st.backward()
    st.sync()
    return st


def run_layer_by_layer(H, sc, params, others, x, dy, nstreams):
    """One LayerBuffers per block, forward calls in order, backward calls in reverse, a device-wide wait
    between calls; returns per-block device tensors in the stack's layout."""
    n = len(params)
    bufs = []
    cur = x
    for l in range(n):
        b = H.LayerBuffers(sc, params[l], cur, dy, others[l], nstreams=nstreams)
        b.forward()
        b.sync()
        bufs.append(b)
        cur = b.y.to("cpu", torch.float32).numpy()          # exact: bf16 values widened
    for l in reversed(range(n)):
        b = bufs[l]
        if l < n - 1:
            b.dy.copy_(bufs[l + 1].dx)
            b.sync()
        b.backward()
        b.sync()
    return bufs


@pytest.mark.parametrize("base,nlayers,p,q,nstreams", [
    ("tiny", 3, 2, 2, 4), ("tiny", 2, 4, 2, 8), ("tiny", 2, 4, 1, 2), ("tiny-llama", 3, 2, 2, 4),
    ("tiny-llama", 2, 1, 4, 1),
    # more than two slices: the weight gradients of a block are one launch per matrix over all rows, and from the third
    # block on the tensors those launches read, kept twice and used in turn, come round again
    ("tiny", 5, 4, 2, 4), ("tiny-llama", 4, 4, 2, 4), ("tiny", 4, 4, 1, 3), ("tiny", 3, 4, 2, 1)])
def test_stack_is_bitwise_the_blocks_called_one_by_one(H, base, nlayers, p, q, nstreams):
    stack_against_single_blocks(H, synth.WORKLOADS[base].replace(p=p, q=q, batch=4), nlayers, nstreams)


@pytest.mark.parametrize("base", ["tiny", "tiny-llama"])
def test_stack_with_weight_gradients_slice_by_slice(H, base):
    """cfg.wgrad_per_slice with four slices over four blocks: slices run on from block to block without meeting."""
    stack_against_single_blocks(H, synth.WORKLOADS[base].replace(p=4, q=2, batch=4, wgrad_per_slice=1), 4, 4)


def stack_against_single_blocks(H, sc, nlayers, nstreams):
    from paper_2409_15241_amd import domino
    params, others = synth.make_stack(sc, nlayers, random_affine=True)
    x, dy = synth.make_activations(sc)
    st = run_stack(H, sc, params, others, x, dy, nstreams)
    bufs = run_layer_by_layer(H, sc, params, others, x, dy, nstreams)
    for l, b in enumerate(bufs):
        for k in OUT_KEYS:
            assert torch.equal(st.out[l][k], getattr(b, k)), (l, k)
        for name in SAVED_NAMES:                                # the named tensors; padding between them is unwritten
            if name.startswith("mean") and sc.arch == synth.ARCH_LLAMA:
                continue                                            # RMSNorm keeps no mean
            off, size = domino.domino_saved_slot(st.cfg, name)
            assert torch.equal(st.out[l]["saved"][off:off + size], b.saved[off:off + size]), (l, name)
        for k, g in b.grads.items():
            if g is not None:
                assert torch.equal(st.grads[l][k], g), (l, k)
    assert torch.equal(st.dx, bufs[0].dx)


@pytest.mark.parametrize("base", ["tiny", "tiny-llama"])
def test_stack_parity_with_the_oracle(H, base):
    sc = synth.WORKLOADS[base]
    nlayers = 3
    params, others = synth.make_stack(sc, nlayers, random_affine=True)
    x, dy = synth.make_activations(sc)
    st = run_stack(H, sc, params, others, x, dy, 4)
    Ps = [f64(P) for P in params]
    oth = [f64(o) for o in others]
    F = O.rank_stack_fwd(sc, Ps, x.astype(np.float64), oth)
    B = O.rank_stack_bwd(sc, Ps, F, dy.astype(np.float64), oth)
    worst = {}
    for l in range(nlayers):
        for k in ("attn_partial", "mlp_partial", "y"):
            worst[(l, k)] = relerr(H.to_host_f64(st.out[l][k]), F[l][k])
        for k in ("dln2_partial", "dln1_partial"):
            worst[(l, k)] = relerr(H.to_host_f64(st.out[l][k]), B[l][k])
        for k, g in B[l]["grads"].items():
            if g is not None:
                worst[(l, "d" + k)] = relerr(st.grads[l][k].cpu().numpy().astype(np.float64), g)
    worst["dx"] = relerr(H.to_host_f64(st.dx), B[0]["dx"])
    bad = {k: v for k, v in worst.items() if not v <= TOL}
    assert not bad, f"over tolerance: {bad}"


def test_stack_accumulates_and_repeats_bitwise(H):
    """Two backward passes with accumulate give twice the gradients; a repeated forward + backward gives
    the same bits (the order of every sum is fixed)."""
    sc = synth.WORKLOADS["tiny"].replace(p=2, q=2, batch=4)
    params, others = synth.make_stack(sc, 2, random_affine=True)
    x, dy = synth.make_activations(sc)
    st = run_stack(H, sc, params, others, x, dy, 4)
    first = [{k: (None if g is None else g.clone()) for k, g in G.items()} for G in st.grads]
    dx = st.dx.clone()
    st.forward()
    st.backward()
    st.sync()
    assert torch.equal(dx, st.dx)
    for G0, G1 in zip(first, st.grads):
        for k, g in G0.items():
            if g is not None:
                assert torch.equal(g, G1[k]), k
    st.backward(accumulate=True)
    st.sync()
    for G0, G1 in zip(first, st.grads):                 # (g + s0) + s1 against 2 * (s0 + s1): equal up to fp32 rounding
        for k, g in G0.items():
            if g is not None:
                assert float((G1[k] - 2 * g).abs().max()) <= 1e-5 * float(g.abs().max()), k


def test_deep_stack_of_mid_size_blocks_repeats_bitwise(H):
    """Five blocks of a shape whose kernels take long enough to overlap across streams, four slices on four streams:
    ten passes over the same buffers leave the bits of the first, and those are the bits of the blocks called one by
    one.  (A launch that read a tensor while the block two below already overwrote it would show here.)"""
    sc = synth.ShardConfig("mid-gpt-d64-stack", 1024, 16, 2, 0, 4, 2, 4, 256, 4096, synth.ARCH_GPT, index=15)
    nlayers = 5
    params, others = synth.make_stack(sc, nlayers, random_affine=True)
    x, dy = synth.make_activations(sc)
    st = run_stack(H, sc, params, others, x, dy, 4)
    first = [{k: (None if g is None else g.clone()) for k, g in G.items()} for G in st.grads]
    dx = st.dx.clone()
    for rep in range(10):
        st.forward()
        st.backward()
        st.sync()
        assert torch.equal(dx, st.dx), rep
        for l, (G0, G1) in enumerate(zip(first, st.grads)):
            for k, g in G0.items():
                if g is not None:
                    assert torch.equal(g, G1[k]), (rep, l, k)
    bufs = run_layer_by_layer(H, sc, params, others, x, dy, 4)
    for l, b in enumerate(bufs):
        for k, g in b.grads.items():
            if g is not None:
                assert torch.equal(first[l][k], g), (l, k)
    assert torch.equal(dx, bufs[0].dx)


@pytest.mark.parametrize("name", ["gpt3-13b", "llama2-7b"])
def test_full_size_stack_matches_single_blocks_bitwise(H, name):
    """The benchmark's shard (GPT-3 13B, p=4, q=2, 4 streams; four blocks, so that the tensors its merged weight
    gradients read come round again) and a Llama shard (p=2, q=4; two blocks)."""
    sc = synth.WORKLOADS[name]
    params, others = synth.make_stack(sc, 4 if sc.p > 2 else 2)
    x, dy = synth.make_activations(sc)
    st = run_stack(H, sc, params, others, x, dy, 4)
    bufs = run_layer_by_layer(H, sc, params, others, x, dy, 4)
    for l, b in enumerate(bufs):
        for k in OUT_KEYS:
            assert torch.equal(st.out[l][k], getattr(b, k)), (l, k)
        for k, g in b.grads.items():
            if g is not None:
                assert torch.equal(st.grads[l][k], g), (l, k)
    assert torch.equal(st.dx, bufs[0].dx)


@pytest.mark.parametrize("base,p", [
    pytest.param("tiny", 4, marks=pytest.mark.skip(
        reason="instantiating the graph captured from a stack backward with four slices (merged weight gradients) and three "
               "blocks crashed inside the runtime and the cause has not been shown from the host side: the library refuses "
               "such captures (test_capture_of_a_deep_stack_backward_with_merged_weight_gradients_is_refused) and the case "
               "stays off the GPU")),
    ("tiny-llama", 2), ("tiny-per-slice", 4)])
def test_captured_stack_replays_bitwise(H, base, p):
    """A stack of three blocks captured in a HIP graph on streams[0] (pool of 4) and replayed three times with eager
    work in between: every replay leaves the bits of the eager stack.  (Four slices: with cfg.wgrad_per_slice.)"""
    per_slice = base.endswith("-per-slice")
    sc = synth.WORKLOADS[base.replace("-per-slice", "")].replace(p=p, q=2, batch=4, wgrad_per_slice=int(per_slice))
    nlayers = 3
    params, others = synth.make_stack(sc, nlayers, random_affine=True)
    x, dy = synth.make_activations(sc)
    ref = run_stack(H, sc, params, others, x, dy, 4)
    st = H.StackBuffers(sc, params, x, dy, others, nstreams=4)
    st.forward()
    st.backward()
    st.sync()
    s0 = st.streams[0]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s0):
        st.forward()
        st.backward()
    for rep in range(3):
        st.dx.zero_()
        for G in st.grads:
            for g in G.values():
                if g is not None:
                    g.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(s0):
            graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(st.dx, ref.dx), rep
        for l in range(nlayers):
            for k, g in ref.grads[l].items():
                if g is not None:
                    assert torch.equal(st.grads[l][k], g), (rep, l, k)
        ref.forward()
        ref.backward()
        ref.sync()


def test_capture_of_a_deep_stack_backward_with_merged_weight_gradients_is_refused(H):
    """streams[0] under capture, four row slices, two blocks: the stack backward returns DOMINO_ERR_UNSUPPORTED and has
    enqueued nothing, so the capture ends with an empty graph (destroyed, never instantiated)."""
    import ctypes
    from paper_2409_15241_amd import domino as D
    sc = synth.WORKLOADS["tiny"].replace(p=4, q=2, batch=4)
    params, others = synth.make_stack(sc, 2, random_affine=True)
    x, dy = synth.make_activations(sc)
    st = run_stack(H, sc, params, others, x, dy, 4)            # eager: fine
    with open("/proc/self/maps") as fh:
        paths = {ln.split()[-1] for ln in fh if "libamdhip64" in ln}
    assert len(paths) == 1, paths
    hip = ctypes.CDLL(paths.pop())
    s0 = ctypes.c_void_p(st.streams[0].cuda_stream)
    assert hip.hipStreamBeginCapture(s0, 1) == 0              # thread-local capture mode
    code = 0
    try:
        try:
            st.backward()
        except D.DominoError as e:
            code = e.code
    finally:
        graph = ctypes.c_void_p()
        rc = hip.hipStreamEndCapture(s0, ctypes.byref(graph))
        nodes = ctypes.c_size_t(123)
        if rc == 0 and graph:
            hip.hipGraphGetNodes(graph, None, ctypes.byref(nodes))
            hip.hipGraphDestroy(graph)
    assert rc == 0 and code == D.ERR_UNSUPPORTED and "one domino_layer_bwd call per block" in D.domino_last_error()
    assert nodes.value == 0
    st.forward(); st.backward(); st.sync()                     # and the pool is usable afterwards


def test_stack_rejects_bad_arguments(H):
    from paper_2409_15241_amd import domino
    sc = synth.WORKLOADS["tiny"]
    params, others = synth.make_stack(sc, 2)
    x, dy = synth.make_activations(sc)
    st = H.StackBuffers(sc, params, x, dy, others)
    small = st.workspace[: domino.domino_workspace_bytes(st.cfg)]       # one block's workspace only
    io = [dict(attn_partial=b["attn_partial"], mlp_partial=b["mlp_partial"], y=b["y"], saved=b["saved"]) for b in st.out]
    with pytest.raises(domino.DominoError) as e:
        domino.domino_stack_fwd(st.cfg, st.params, st.x, io, small, st.streams)
    assert e.value.code == domino.ERR_WORKSPACE_TOO_SMALL
    io[1]["y"] = None
    with pytest.raises(domino.DominoError) as e:
        domino.domino_stack_fwd(st.cfg, st.params, st.x, io, st.workspace, st.streams)
    assert e.value.code == domino.ERR_NULL_POINTER
    assert domino.domino_stack_workspace_bytes(st.cfg, 0) == 0
    st.sync()
