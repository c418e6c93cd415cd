"""Layer parity: domino_layer_fwd / domino_layer_bwd through the C ABI against the fp64 oracle, on the
same seeded inputs, for every output and every gradient tensor.  Bar (from the benchmark spec):
max|err| <= 2e-2 * max|ref| per tensor, at every p x q slicing."""
import numpy as np
import pytest

from oracle import domino_oracle as O
from paper_2409_15241_amd import synth

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

TOL = 2e-2


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


def run_gpu(H, sc, params, x, dy, others, nstreams=4, accumulate_twice=False):
    buf = H.LayerBuffers(sc, params, x, dy, others, nstreams=nstreams)
    buf.forward()
    buf.backward(accumulate=False)
    if accumulate_twice:
        buf.backward(accumulate=True)
    buf.sync()
    out = {k: H.to_host_f64(getattr(buf, k)) for k in
           ("attn_partial", "mlp_partial", "y", "dln2_partial", "dln1_partial", "dx")}
    out["grads"] = {k: (None if g is None else g.cpu().numpy().astype(np.float64)) for k, g in buf.grads.items()}
    shp = (sc.batch, sc.seq)
    out["x1"] = H.to_host_f64(buf.saved_tensor("x1")).reshape(*shp, sc.hidden)
    out["ctx"] = H.to_host_f64(buf.saved_tensor("ctx")).reshape(*shp, sc.h_local)
    out["lse"] = buf.saved_tensor("lse").cpu().numpy().astype(np.float64).reshape(sc.batch, sc.local_heads, sc.seq)
    # q, k, v as the attention kernel read them (bf16, after the rotary embedding), first and last batch element
    qkv = buf.saved_tensor("qkv").view(sc.batch, sc.seq, 3, sc.local_heads, sc.head_dim)
    picks = sorted({0, sc.batch - 1})
    out["qkv_batches"] = picks
    out["qkv"] = np.stack([H.to_host_f64(qkv[b]) for b in picks]).transpose(2, 0, 3, 1, 4)    # [3, b', heads, s, d]
    return out


def oracle(sc, params, x, dy, others):
    P = f64(params)
    oth = f64(others) if others else {}
    F = O.rank_layer_fwd(sc, P, x.astype(np.float64), oth.get("attn_others"), oth.get("mlp_others"))
    B = O.rank_layer_bwd(sc, P, F, dy.astype(np.float64), oth.get("dln2_others"), oth.get("dln1_others"))
    return F, B


# The softmax statistics, absolute: against the whole-layer oracle the log-sum-exp carries the bf16 rounding of q and k
# (an error that grows with the size of the scores), so the kernel's own statistics are held, at every size, against
# the oracle's attention on exactly the q, k, v the kernel read: there only fp32 summation and the 2^x unit differ.
LSE_ABS_TOL = 2e-3


def check(got, F, B, tol=TOL, grad_scale=1.0):
    worst = {}
    for k in ("attn_partial", "mlp_partial", "y", "x1", "ctx", "lse"):
        worst[k] = relerr(got[k], F[k])
    q, k_, v = got["qkv"]
    ctx2, lse2 = O.attention_fwd(q, k_, v)
    bsel = got["qkv_batches"]
    lse_abs = float(np.max(np.abs(got["lse"][bsel] - lse2)))
    assert lse_abs < LSE_ABS_TOL, f"max |lse error| {lse_abs:.3e} against attention on the kernel's own q, k, v (bar {LSE_ABS_TOL})"
    b, s = got["ctx"].shape[:2]
    ctx_gpu = got["ctx"].reshape(b, s, q.shape[1], q.shape[3])[bsel].transpose(0, 2, 1, 3)
    worst["ctx_own_qkv"] = relerr(ctx_gpu, ctx2)
    assert worst["ctx_own_qkv"] <= 1e-2, worst
    for k in ("dln2_partial", "dln1_partial", "dx"):
        worst[k] = relerr(got[k], B[k])
    for k, g in B["grads"].items():
        if g is None:
            assert got["grads"][k] is None
        else:
            worst["d" + k] = relerr(got["grads"][k], grad_scale * g)
    bad = {k: v for k, v in worst.items() if not v <= tol}
    assert not bad, f"over tolerance: {bad}\nall: {worst}"
    return worst


_ORACLE_CACHE = {}     # the last workload's inputs and oracle result: it does not depend on p, q or the pool


def case(H, sc, random_affine=False, with_others=True, nstreams=4):
    """One forward + backward through the C ABI against the oracle.  The oracle result depends on the shard, not on
    the slicing, so consecutive cases that differ in (p, q, streams) only share one oracle run."""
    key = (sc.replace(p=1, q=1, wgrad_per_slice=0), random_affine, with_others)
    if key not in _ORACLE_CACHE:
        _ORACLE_CACHE.clear()
        params = synth.make_rank_params(sc, random_affine=random_affine)
        x, dy = synth.make_activations(sc)
        others = synth.make_others(sc) if with_others else None
        _ORACLE_CACHE[key] = (params, x, dy, others) + oracle(sc, params, x, dy, others)
    params, x, dy, others, F, B = _ORACLE_CACHE[key]
    got = run_gpu(H, sc, params, x, dy, others, nstreams)
    return check(got, F, B)


TINY = synth.WORKLOADS["tiny"]
TINYL = synth.WORKLOADS["tiny-llama"]


@pytest.mark.parametrize("base", [TINY, TINYL], ids=["gpt", "llama"])
@pytest.mark.parametrize("p,q", [(1, 1), (2, 1), (1, 2), (2, 2), (1, 4), (2, 4), (4, 1), (4, 2), (4, 4), (8, 1), (8, 2),
                                 (1, 8)])
def test_tiny_every_slicing(H, base, p, q):
    sc = base.replace(p=p, q=q, batch=p if p >= 4 else base.batch)
    case(H, sc, random_affine=True)


@pytest.mark.parametrize("base", [TINY, TINYL], ids=["gpt", "llama"])
@pytest.mark.parametrize("p,q,nstreams", [(4, 2, 4), (4, 1, 2), (8, 2, 4), (4, 4, 8)])
def test_tiny_weight_gradients_slice_by_slice_for_more_than_two_slices(H, base, p, q, nstreams):
    """cfg.wgrad_per_slice: the order of Sec. 4.1.2 (a slice's weight gradient right behind its input gradient, summed
    over the slices in slice order) instead of one launch per matrix over all rows."""
    sc = base.replace(p=p, q=q, batch=p, wgrad_per_slice=1)
    case(H, sc, random_affine=True, nstreams=nstreams)


@pytest.mark.parametrize("base", [TINY, TINYL], ids=["gpt", "llama"])
def test_tiny_as_configured_zero_biases_no_others(H, base):
    case(H, base, random_affine=False, with_others=False)


@pytest.mark.parametrize("rank", [0, 1])
def test_tiny_other_rank_and_erf_gelu(H, rank):
    case(H, TINY.replace(rank=rank, gelu_tanh=0), random_affine=True)


def test_ranks_sum_to_the_unsharded_layer(H):
    """The library is called once per rank on the same GPU; with the true 'others' (from the oracle's
    simulated all-reduces) each rank's y equals the full layer's, and the partials sum to the
    unsharded sub-layer outputs (Eq. 1)."""
    sc = TINY
    shards = [synth.make_rank_params(sc, r, random_affine=True) for r in range(sc.tp)]
    x, dy = synth.make_activations(sc)
    fwd, bwd = O.simulate_tp(sc, [f64(s) for s in shards], x.astype(np.float64), dy.astype(np.float64))
    full = O.full_from_shards([f64(s) for s in shards], sc)
    Ff = O.full_layer_fwd(sc, full, x.astype(np.float64))
    Bf = O.full_layer_bwd(sc, full, Ff, dy.astype(np.float64))
    rb = synth.round_bf16
    attn_sum, mlp_sum, d2_sum, d1_sum = 0, 0, 0, 0
    for r in range(sc.tp):
        others = {
            "attn_others": rb((Ff["attn_partial"] - fwd[r]["attn_partial"]).astype(np.float32)),
            "mlp_others": rb((Ff["mlp_partial"] - fwd[r]["mlp_partial"]).astype(np.float32)),
            "dln2_others": rb((Bf["dln2_partial"] - bwd[r]["dln2_partial"]).astype(np.float32)),
            "dln1_others": rb((Bf["dln1_partial"] - bwd[r]["dln1_partial"]).astype(np.float32)),
        }
        got = run_gpu(H, sc.replace(rank=r), shards[r], x, dy, others)
        assert relerr(got["y"], Ff["y"]) < TOL
        assert relerr(got["dx"], Bf["dx"]) < TOL
        attn_sum = attn_sum + got["attn_partial"]; mlp_sum = mlp_sum + got["mlp_partial"]
        d2_sum = d2_sum + got["dln2_partial"]; d1_sum = d1_sum + got["dln1_partial"]
    assert relerr(attn_sum, Ff["attn_partial"]) < TOL
    assert relerr(mlp_sum, Ff["mlp_partial"]) < TOL
    assert relerr(d2_sum, Bf["dln2_partial"]) < TOL
    assert relerr(d1_sum, Bf["dln1_partial"]) < TOL


MID = [
    # head_dim 80, out-projection K = 320, sequence not a multiple of the 128-query block
    synth.ShardConfig("mid-gpt-d80", 640, 8, 2, 1, 2, 2, 2, 328, 2560, synth.ARCH_GPT, index=11),
    # head_dim 128, SwiGLU width 43*32 = 1376 (K tail of half a tile), q = 4
    synth.ShardConfig("mid-llama", 1024, 8, 4, 2, 1, 4, 2, 200, 5504, synth.ARCH_LLAMA, index=12),
    # head_dim 64 with a 256x256-tile sized problem
    synth.ShardConfig("mid-gpt-d64", 1024, 16, 2, 0, 2, 1, 4, 256, 4096, synth.ARCH_GPT, index=13),
    # rotary embedding on heads of 80 columns (a separate pass over q and k in the forward) and of 64 columns (in the
    # QKV product's epilogue, like the heads of 128 of mid-llama), sequences that end inside a tile
    synth.ShardConfig("mid-llama-d80", 640, 8, 2, 1, 2, 2, 2, 136, 1792, synth.ARCH_LLAMA, index=15),
    synth.ShardConfig("mid-llama-d64", 512, 8, 2, 0, 2, 1, 4, 72, 1536, synth.ARCH_LLAMA, index=16),
]


@pytest.mark.parametrize("sc", MID, ids=[m.name for m in MID])
def test_mid_shapes_with_ragged_tiles(H, sc):
    case(H, sc, random_affine=True)


# head_dim 128 at hidden 8192: the widest rows the norm kernels take (1024 threads a row in the backward, with the
# column sums of the two row-cut products' bias gradients)
WIDE = synth.ShardConfig("wide-gpt-h8192", 8192, 64, 8, 3, 2, 2, 2, 136, 32768, synth.ARCH_GPT, index=14)


def test_widest_hidden_size(H):
    case(H, WIDE, random_affine=True)


# the five configured shards (GPT-3 13B is the one bench.py times) and shards at the evaluation's own shapes
FULL = [synth.WORKLOADS[n] for n in ("gpt3-13b", "gpt3-2.7b", "llama2-7b", "llama2-13b", "gpt3-30b", "gpt3-2.7b-s512-mb64",
                                     "llama2-13b-s512-mb16")]


@pytest.mark.parametrize("sc", FULL, ids=[m.name for m in FULL])
def test_full_size_shard_in_the_benchmark_configuration(H, sc):
    """The configured full-size shards (GPT-3 13B is the one bench.py times), on 4 streams as bench.py
    launches them: every output and gradient element against the oracle, which finishes a full-size
    layer in seconds."""
    case(H, sc, random_affine=True, nstreams=4)


# Other slicings of full-size shards: the tile of every product is chosen from the rows of a slice and from the
# number of slices in flight, so each (p, q, pool) runs other kernel instantiations than the configured one.
SLICINGS = [("gpt3-13b", 1, 1, 1), ("gpt3-13b", 2, 4, 2), ("gpt3-13b", 4, 1, 4), ("gpt3-13b", 2, 2, 4),
            ("llama2-7b", 1, 1, 1), ("llama2-7b", 2, 1, 2), ("llama2-7b", 1, 4, 4)]


@pytest.mark.parametrize("name,p,q,nstreams", SLICINGS, ids=[f"{n}-p{p}q{q}-{k}streams" for n, p, q, k in SLICINGS])
def test_full_size_shard_at_other_slicings(H, name, p, q, nstreams):
    case(H, synth.WORKLOADS[name].replace(p=p, q=q), random_affine=True, nstreams=nstreams)


def test_full_size_shard_with_weight_gradients_slice_by_slice(H):
    """The benchmark's shard as configured (p=4, q=2, 4 streams) in the order of Sec. 4.1.2 (cfg.wgrad_per_slice)."""
    case(H, synth.WORKLOADS["gpt3-13b"].replace(wgrad_per_slice=1), random_affine=True, nstreams=4)


def test_schedule_invariance_bitwise(H):
    """The same call on 1 stream and on 4 streams: identical bits (accumulation order is fixed)."""
    sc = TINY.replace(batch=4, p=4, q=2)
    params = synth.make_rank_params(sc, random_affine=True)
    x, dy = synth.make_activations(sc)
    others = synth.make_others(sc)
    a = run_gpu(H, sc, params, x, dy, others, nstreams=1)
    b = run_gpu(H, sc, params, x, dy, others, nstreams=4)
    c = run_gpu(H, sc, params, x, dy, others, nstreams=8)
    _same_bits(a, b, c)
    # ... and so does the slice-by-slice order of the weight gradients (its sums differ from the merged ones in rounding only)
    ps = sc.replace(wgrad_per_slice=1)
    a2 = run_gpu(H, ps, params, x, dy, others, nstreams=1)
    _same_bits(a2, run_gpu(H, ps, params, x, dy, others, nstreams=4), run_gpu(H, ps, params, x, dy, others, nstreams=8))
    for k, g in a["grads"].items():
        if g is not None:
            np.testing.assert_allclose(a2["grads"][k], g, rtol=0, atol=1e-5 * float(np.abs(g).max()), err_msg=k)


def _same_bits(a, b, c):
    for k in ("attn_partial", "mlp_partial", "y", "dln2_partial", "dln1_partial", "dx"):
        np.testing.assert_array_equal(a[k], b[k], err_msg=k)
        np.testing.assert_array_equal(a[k], c[k], err_msg=k)
    for k, g in a["grads"].items():
        if g is not None:
            np.testing.assert_array_equal(g, b["grads"][k], err_msg=k)
            np.testing.assert_array_equal(g, c["grads"][k], err_msg=k)


# GeLU at head_dim 64, SwiGLU + rotary embedding at head_dim 128 (batch 4 so that two slices run side by side), and
# head_dim 80
REPEAT = [(MID[2], 2), (MID[2], 4), (MID[1].replace(batch=4, p=2), 2), (MID[0], 2)]


@pytest.mark.parametrize("sc,nstreams", REPEAT, ids=[f"{c.name}-{k}streams" for c, k in REPEAT])
def test_repeated_steps_are_bitwise_identical(H, sc, nstreams):
    """The same step on the same buffers, many times while other slices' kernels share the CUs: every
    repetition gives the bits of the first (no value may depend on the timing of a look-ahead read or
    of another stream)."""
    params = synth.make_rank_params(sc, random_affine=True)
    x, dy = synth.make_activations(sc)
    buf = H.LayerBuffers(sc, params, x, dy, synth.make_others(sc), nstreams=nstreams)
    first = None
    for rep in range(40):
        buf.forward()
        buf.backward(accumulate=False)
        buf.sync()
        cur = {k: g.clone() for k, g in buf.grads.items() if g is not None}
        cur.update(y=buf.y.clone(), dx=buf.dx.clone(), dln1=buf.dln1_partial.clone(), dln2=buf.dln2_partial.clone())
        if first is None:
            first = cur
            continue
        diff = [k for k in cur if not torch.equal(cur[k], first[k])]
        assert not diff, f"repetition {rep} differs from the first in {diff}"


def test_accumulate_adds_to_existing_gradients(H):
    sc = TINY
    params = synth.make_rank_params(sc, random_affine=True)
    x, dy = synth.make_activations(sc)
    got = run_gpu(H, sc, params, x, dy, None, accumulate_twice=True)
    F, B = oracle(sc, params, x, dy, None)
    check(got, F, B, grad_scale=2.0)


def test_grid_search_returns_a_measured_setting(H):
    from paper_2409_15241_amd import tune
    best, table = tune.tune(TINY, pairs=[(1, 1), (2, 2)], streams=(1, 2), steps=2, warmup=1)
    assert best in table and best[3] > 0.0
    assert {(p, q) for p, q, _, _ in table} == {(1, 1), (2, 2)}


def test_profile_records_give_the_timeline_of_a_step(H):
    """Every launch of a profiled step comes back with its step class, the pool stream it ran on and times that
    are ordered on each stream; the per-class sums of domino_profile_read are the sums of these records."""
    from paper_2409_15241_amd import domino as D
    sc = TINY.replace(batch=4, p=4, q=2)
    params = synth.make_rank_params(sc, random_affine=True)
    x, dy = synth.make_activations(sc)
    buf = H.LayerBuffers(sc, params, x, dy, synth.make_others(sc), nstreams=4)
    buf.forward(); buf.backward(); buf.sync()
    D.domino_profile_reset()
    D.domino_profile_enable(True)
    try:
        buf.forward(); buf.backward(); buf.sync()
    finally:
        D.domino_profile_enable(False)
    n = D.domino_profile_records()
    recs = [D.domino_profile_record(i) for i in range(n)]
    assert n == sum(D.domino_profile_read(c)[1] for c in range(D.domino_profile_classes())) > 40
    handles = {s.cuda_stream for s in buf.streams}
    last = {}
    for name, st, a, b in recs:
        assert st in handles and b >= a
        assert a >= last.get(st, -1e9)           # enqueue order is execution order on a stream
        last[st] = b
    for c in range(D.domino_profile_classes()):
        tot, cnt = D.domino_profile_read(c)
        mine = [b - a for name, _, a, b in recs if name == D.domino_profile_name(c)]
        assert cnt == len(mine) and abs(tot - sum(mine)) <= 1e-3 * max(tot, 1e-3)
    with pytest.raises(D.DominoError) as e:
        D.domino_profile_record(n)
    assert e.value.code == D.ERR_INVALID_ARG
    D.domino_profile_reset()
    assert D.domino_profile_records() == 0


def test_two_host_threads_with_their_own_pools(H):
    """Two host threads enqueue steps at the same time, each on its own buffers and stream pool: the library
    serialises the enqueueing (one mutex, one event pool per device) and every result has the bits of a
    single-threaded run."""
    import threading
    sc = TINY.replace(batch=4, p=2, q=2)
    params = synth.make_rank_params(sc, random_affine=True)
    x, dy = synth.make_activations(sc)
    others = synth.make_others(sc)
    ref = run_gpu(H, sc, params, x, dy, others, nstreams=2)
    bufs = [H.LayerBuffers(sc, params, x, dy, others, nstreams=2) for _ in range(2)]
    errors = []

    def work(buf):
        try:
            for _ in range(25):
                buf.forward()
                buf.backward(accumulate=False)
            buf.sync()
        except Exception as e:          # noqa: BLE001
            errors.append(e)

    threads = [threading.Thread(target=work, args=(b,)) for b in bufs]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not errors and not any(t.is_alive() for t in threads)
    for b in bufs:
        np.testing.assert_array_equal(H.to_host_f64(b.y), ref["y"])
        np.testing.assert_array_equal(H.to_host_f64(b.dx), ref["dx"])
        for k, g in b.grads.items():
            if g is not None:
                np.testing.assert_array_equal(g.cpu().numpy(), ref["grads"][k], err_msg=k)


@pytest.mark.parametrize("per_slice", [0, 1], ids=["", "wgrads-slice-by-slice"])
@pytest.mark.parametrize("p,nstreams", [(4, 4), (2, 4), (1, 2), (2, 2), (4, 1)],
                         ids=["4slices-4streams", "2slices-4streams", "1slice-2streams", "2slices-2streams", "4slices-1stream"])
def test_graph_replay_is_bitwise_the_eager_step(H, p, nstreams, per_slice):
    """The step captured once in a HIP graph on streams[0] (the library forks and joins the pool inside the capture,
    allocates nothing and records no memset) and replayed several times, with eager steps and synchronisations in
    between: every replay leaves the bits of the eager step.  (With twice as many streams as slices an eager backward
    runs the weight gradients on streams of their own; a captured one keeps them on the slices' streams.)"""
    if per_slice and p <= 2:
        pytest.skip("cfg.wgrad_per_slice changes nothing for one or two slices")
    sc = TINY.replace(batch=4, p=p, q=2, wgrad_per_slice=per_slice)
    params = synth.make_rank_params(sc, random_affine=True)
    x, dy = synth.make_activations(sc)
    others = synth.make_others(sc)
    ref = run_gpu(H, sc, params, x, dy, others, nstreams=1)
    buf = H.LayerBuffers(sc, params, x, dy, others, nstreams=nstreams)
    other = H.LayerBuffers(sc, params, x, dy, others, nstreams=nstreams)       # eager work between the replays

    def step():
        buf.forward()
        buf.backward(accumulate=False)

    step()
    buf.sync()
    s0 = buf.streams[0]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s0):
        step()
    for rep in range(4):
        for t in (buf.y, buf.dx, buf.attn_partial, buf.mlp_partial, buf.dln1_partial, buf.dln2_partial):
            t.zero_()
        for g in buf.grads.values():
            if g is not None:
                g.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(s0):
            graph.replay()
        torch.cuda.synchronize()
        for k in ("attn_partial", "mlp_partial", "y", "dln2_partial", "dln1_partial", "dx"):
            np.testing.assert_array_equal(H.to_host_f64(getattr(buf, k)), ref[k], err_msg=f"replay {rep}: {k}")
        for k, g in buf.grads.items():
            if g is not None:
                np.testing.assert_array_equal(g.cpu().numpy(), ref["grads"][k], err_msg=f"replay {rep}: {k}")
        other.forward()
        other.backward(accumulate=False)
        other.sync()


def _hip_runtime():
    """The HIP runtime this process already runs on (torch's), for the few calls the test below makes itself."""
    import ctypes
    with open("/proc/self/maps") as fh:
        paths = {ln.split()[-1] for ln in fh if "libamdhip64" in ln}
    assert len(paths) == 1, paths
    return ctypes.CDLL(paths.pop())


def test_capture_with_an_unsupported_pool_is_refused_before_anything_is_enqueued(H):
    """streams[0] under capture with a pool of 3 streams: the call returns DOMINO_ERR_UNSUPPORTED and has enqueued
    nothing, so the capture ends with an empty graph (which is destroyed, never instantiated)."""
    import ctypes
    from paper_2409_15241_amd import domino as D
    sc = TINY.replace(batch=4, p=4, q=2)
    params = synth.make_rank_params(sc, random_affine=True)
    x, dy = synth.make_activations(sc)
    buf = H.LayerBuffers(sc, params, x, dy, synth.make_others(sc), nstreams=3)
    buf.forward(); buf.backward(); buf.sync()                  # eager calls on 3 streams are fine
    hip = _hip_runtime()
    s0 = ctypes.c_void_p(buf.streams[0].cuda_stream)
    assert hip.hipStreamBeginCapture(s0, 1) == 0              # thread-local capture mode
    codes = []
    try:
        for fn in (buf.forward, buf.backward):
            try:
                fn()
                codes.append(0)
            except D.DominoError as e:
                codes.append(e.code)
    finally:
        graph = ctypes.c_void_p()
        rc = hip.hipStreamEndCapture(s0, ctypes.byref(graph))
        nodes = ctypes.c_size_t(123)
        if rc == 0 and graph:
            hip.hipGraphGetNodes(graph, None, ctypes.byref(nodes))
            hip.hipGraphDestroy(graph)
    assert rc == 0 and codes == [D.ERR_UNSUPPORTED, D.ERR_UNSUPPORTED]
    assert nodes.value == 0
    buf.forward(); buf.backward(); buf.sync()                  # and the pool is usable afterwards


@pytest.mark.parametrize("nstreams", [3, 8])
@pytest.mark.skip(reason="instantiating a HIP graph captured with a pool of 3 or 8 streams aborted inside the runtime and the "
                         "cause has not been shown from the host side: the library refuses such captures "
                         "(test_capture_with_an_unsupported_pool_is_refused...) and the case stays off the GPU")
def test_graph_replay_with_other_pools(H, nstreams):
    sc = TINY.replace(batch=4, p=4, q=2)
    params = synth.make_rank_params(sc, random_affine=True)
    x, dy = synth.make_activations(sc)
    buf = H.LayerBuffers(sc, params, x, dy, synth.make_others(sc), nstreams=nstreams)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=buf.streams[0]):
        buf.forward()
        buf.backward(accumulate=False)
    graph.replay()
    buf.sync()


def test_hardware_queue_note(H, hw_queues_at_start):
    """Four slices on four streams with fewer hardware queues than streams + 1 configured: the library says so
    once; with enough queues it stays silent."""
    from paper_2409_15241_amd import domino as D
    sc = TINY.replace(batch=4, p=4, q=2)
    params = synth.make_rank_params(sc, random_affine=True)
    x, dy = synth.make_activations(sc)
    buf = H.LayerBuffers(sc, params, x, dy, synth.make_others(sc), nstreams=4)
    buf.forward(); buf.sync()
    note = D.domino_last_warning()
    if hw_queues_at_start >= 5:
        assert note == ""
    else:
        assert "GPU_MAX_HW_QUEUES" in note and ">= 5" in note
