"""Parity of each HIP kernel with the matching oracle function, through the C ABI, at shapes that span
several tiles and end in ragged tails.  Bar for whole tensors: max|err| <= 2e-2 * max|ref| (bf16 inputs,
fp32 accumulation); the single kernels are held to tighter bounds derived from one bf16 rounding of
the output (2^-9 relative) so that an indexing slip cannot hide inside the layer tolerance."""
import math

import numpy as np
import pytest

from oracle import domino_oracle as O
from paper_2409_15241_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def dom():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2409_15241_amd import domino
    domino.load()
    return domino


def rnd(rng, shape, std=1.0):
    return synth.round_bf16((rng.standard_normal(shape) * std).astype(np.float32))


def dev(a):
    from paper_2409_15241_amd.harness import to_device_bf16
    return to_device_bf16(a)


def host(t):
    return t.detach().to("cpu", torch.float32).numpy().astype(np.float64)


def relerr(got, ref):
    return float(np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-30))


BF16_OUT = 6e-3     # one output rounding (2^-9 = 2e-3) plus bf16-rounded intermediates feeding nonlinearities
SHAPES = [(328, 200, 328), (256, 256, 64), (520, 776, 1376), (64, 2752 // 2, 192), (8, 8, 8)]   # last: the smallest legal problem


@pytest.mark.parametrize("tile", [0, 1, 2, 3])
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_nn_store_bias(dom, tile, M, N, K):
    rng = np.random.default_rng(M * 7 + N * 3 + K + tile)
    A, B, bias = rnd(rng, (M, K)), rnd(rng, (K, N), 0.05), rnd(rng, (N,), 0.5)
    Cd = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    dom.domino_gemm(dom.GEMM_NN, dom.EPI_STORE, tile, dev(A), K, dev(B), N, Cd, N, M, N, K, bias=dev(bias))
    torch.cuda.synchronize()
    ref = A.astype(np.float64) @ B.astype(np.float64) + bias
    assert relerr(host(Cd), ref) < BF16_OUT


def test_gemm_nn_writes_a_column_slice_in_place(dom):
    """(XA) * B_j of Eq. 4: B is a column view (ldb > N), C lands inside a wider buffer (ldc > N)."""
    rng = np.random.default_rng(5)
    M, K, H, q = 264, 136, 512, 4
    A, B = rnd(rng, (M, K)), rnd(rng, (K, H), 0.05)
    Cd = torch.full((M, H), 7.0, dtype=torch.bfloat16, device="cuda")
    Bd = dev(B)
    w = H // q
    for j in (2, 0):
        dom.domino_gemm(dom.GEMM_NN, dom.EPI_STORE, -1, dev(A), K, Bd[:, j * w:], H, Cd[:, j * w:], H, M, w, K)
    torch.cuda.synchronize()
    got = host(Cd)
    ref = A.astype(np.float64) @ B.astype(np.float64)
    for j in range(q):
        if j in (0, 2):
            assert relerr(got[:, j * w:(j + 1) * w], ref[:, j * w:(j + 1) * w]) < BF16_OUT
        else:
            assert np.all(got[:, j * w:(j + 1) * w] == 7.0)        # untouched neighbours


@pytest.mark.parametrize("tanh", [1, 0])
@pytest.mark.parametrize("tile", [0, 2, 3])
def test_gemm_nn_bias_gelu(dom, tile, tanh):
    rng = np.random.default_rng(11 + tile)
    M, N, K = 328, 264, 200
    A, B, bias = rnd(rng, (M, K)), rnd(rng, (K, N), 0.08), rnd(rng, (N,), 0.3)
    Cd = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    pre = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    dom.domino_gemm(dom.GEMM_NN, dom.EPI_BIAS_GELU, tile, dev(A), K, dev(B), N, Cd, N, M, N, K, bias=dev(bias),
                    aux=pre, ldaux=N, gelu_tanh=tanh)
    torch.cuda.synchronize()
    ref_pre = A.astype(np.float64) @ B.astype(np.float64) + bias
    assert relerr(host(pre), ref_pre) < BF16_OUT
    assert relerr(host(Cd), O.gelu(ref_pre, bool(tanh))) < BF16_OUT


@pytest.mark.parametrize("tile", [0, 1, 2, 3])
@pytest.mark.parametrize("fl", [352, 96, 1376])
def test_gemm_nn_swiglu(dom, tile, fl):
    rng = np.random.default_rng(13 + tile + fl)
    M, K = 200, 136
    A, B = rnd(rng, (M, K)), rnd(rng, (K, 2 * fl), 0.1)
    act = torch.zeros((M, fl), dtype=torch.bfloat16, device="cuda")
    gu = torch.zeros((M, 2 * fl), dtype=torch.bfloat16, device="cuda")
    dom.domino_gemm(dom.GEMM_NN, dom.EPI_SWIGLU, tile, dev(A), K, dev(B), 2 * fl, act, fl, M, fl, K,
                    aux=gu, ldaux=2 * fl, n_split=fl)
    torch.cuda.synchronize()
    ref = A.astype(np.float64) @ B.astype(np.float64)
    assert relerr(host(gu), ref) < BF16_OUT
    assert relerr(host(act), O.silu(ref[:, :fl]) * ref[:, fl:]) < BF16_OUT


@pytest.mark.parametrize("tile", [0, 1, 2, 3])
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_nt_input_gradient(dom, tile, M, N, K):
    rng = np.random.default_rng(M + N + K + 17 * tile)
    A, B = rnd(rng, (M, K)), rnd(rng, (N, K), 0.05)
    Cd = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    dom.domino_gemm(dom.GEMM_NT, dom.EPI_STORE, tile, dev(A), K, dev(B), K, Cd, N, M, N, K)
    torch.cuda.synchronize()
    assert relerr(host(Cd), A.astype(np.float64) @ B.astype(np.float64).T) < BF16_OUT


@pytest.mark.parametrize("tanh", [1, 0])
def test_gemm_nt_gelu_backward(dom, tanh):
    rng = np.random.default_rng(19)
    M, N, K = 264, 328, 136
    A, B, pre = rnd(rng, (M, K)), rnd(rng, (N, K), 0.05), rnd(rng, (M, N), 1.5)
    Cd = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    dom.domino_gemm(dom.GEMM_NT, dom.EPI_DGELU, -1, dev(A), K, dev(B), K, Cd, N, M, N, K, aux=dev(pre), ldaux=N,
                    gelu_tanh=tanh)
    torch.cuda.synchronize()
    ref = (A.astype(np.float64) @ B.astype(np.float64).T) * O.gelu_grad(pre.astype(np.float64), bool(tanh))
    assert relerr(host(Cd), ref) < BF16_OUT


def test_gemm_nt_swiglu_backward(dom):
    rng = np.random.default_rng(23)
    M, fl, K = 200, 352, 136
    A, B, gu = rnd(rng, (M, K)), rnd(rng, (fl, K), 0.05), rnd(rng, (M, 2 * fl), 1.5)
    Cd = torch.zeros((M, 2 * fl), dtype=torch.bfloat16, device="cuda")
    dom.domino_gemm(dom.GEMM_NT, dom.EPI_DSWIGLU, -1, dev(A), K, dev(B), K, Cd, 2 * fl, M, fl, K, aux=dev(gu),
                    ldaux=2 * fl, n_split=fl)
    torch.cuda.synchronize()
    d_act = A.astype(np.float64) @ B.astype(np.float64).T
    g, u = gu[:, :fl].astype(np.float64), gu[:, fl:].astype(np.float64)
    ref = np.concatenate([d_act * u * O.silu_grad(g), d_act * O.silu(g)], axis=1)
    assert relerr(host(Cd), ref) < BF16_OUT


@pytest.mark.parametrize("tile", [0, 1, 2, 3])
@pytest.mark.parametrize("M,N,K", [(328, 200, 328), (640, 520, 2048), (136, 1376, 264)])
def test_gemm_tn_weight_gradient_accumulates(dom, tile, M, N, K):
    rng = np.random.default_rng(M + 2 * N + 3 * K + tile)
    A, B = rnd(rng, (K, M)), rnd(rng, (K, N))
    C0 = rng.standard_normal((M, N)).astype(np.float32)
    Cd = torch.from_numpy(C0.copy()).cuda()
    ref = A.astype(np.float64).T @ B.astype(np.float64)
    dom.domino_gemm(dom.GEMM_TN, dom.EPI_ACC_F32, tile, dev(A), M, dev(B), N, Cd, N, M, N, K, beta=0)
    torch.cuda.synchronize()
    assert relerr(Cd.cpu().numpy().astype(np.float64), ref) < 1e-4
    dom.domino_gemm(dom.GEMM_TN, dom.EPI_ACC_F32, tile, dev(A), M, dev(B), N, Cd, N, M, N, K, beta=1)
    torch.cuda.synchronize()
    assert relerr(Cd.cpu().numpy().astype(np.float64), 2 * ref) < 1e-4


@pytest.mark.parametrize("rms", [0, 1])
@pytest.mark.parametrize("h", [8, 256, 2560, 4096, 5120, 8192])      # 8 and 8192: the narrowest and widest rows accepted
def test_norm_forward(dom, rms, h):
    rng = np.random.default_rng(h + rms)
    rows, eps = 37, 1e-5
    x, a1, a2 = rnd(rng, (rows, h)), rnd(rng, (rows, h), 0.5), rnd(rng, (rows, h), 0.5)
    vec, g = rnd(rng, (h,), 0.1), synth.round_bf16(1 + rnd(rng, (h,), 0.1))
    b = None if rms else rnd(rng, (h,), 0.1)
    y = torch.zeros((rows, h), dtype=torch.bfloat16, device="cuda")
    xs = torch.zeros((rows, h), dtype=torch.bfloat16, device="cuda")
    mean = torch.zeros(rows, dtype=torch.float32, device="cuda")
    rstd = torch.zeros(rows, dtype=torch.float32, device="cuda")
    # plain
    dom.domino_norm_fwd(dev(x), None, None, None, dev(g), dev(b), None, y, mean, rstd, rows, h, rms, eps)
    torch.cuda.synchronize()
    ry, rmean, rrstd = O.norm_fwd(x.astype(np.float64), g, b, eps, bool(rms))
    assert relerr(host(y), ry) < BF16_OUT
    assert relerr(rstd.cpu().numpy(), rrstd) < 1e-5
    if not rms:
        assert np.max(np.abs(mean.cpu().numpy() - rmean)) < 1e-5
    # fused residual sums
    dom.domino_norm_fwd(dev(x), dev(a1), dev(a2), dev(vec), dev(g), dev(b), xs, y, mean, rstd, rows, h, rms, eps)
    torch.cuda.synchronize()
    total = x.astype(np.float64) + a1 + a2 + vec
    assert relerr(host(xs), total) < 4e-3
    ry, _, _ = O.norm_fwd(total, g, b, eps, bool(rms))
    assert relerr(host(y), ry) < 1e-2


@pytest.mark.parametrize("rms", [0, 1])
@pytest.mark.parametrize("rows,h", [(37, 256), (1100, 2560), (300, 5120), (1, 8), (19, 8192)])
def test_norm_backward(dom, rms, rows, h):
    rng = np.random.default_rng(rows + h + rms)
    eps = 1e-5
    x, ga, gb, dres = rnd(rng, (rows, h)), rnd(rng, (rows, h)), rnd(rng, (rows, h), 0.5), rnd(rng, (rows, h))
    g = synth.round_bf16(1 + rnd(rng, (h,), 0.1))
    _, mean, rstd = O.norm_fwd(x.astype(np.float64), g, None, eps, bool(rms))
    dx = torch.zeros((rows, h), dtype=torch.bfloat16, device="cuda")
    dg = torch.zeros(h, dtype=torch.float32, device="cuda")
    db = torch.zeros(h, dtype=torch.float32, device="cuda")
    scratch = torch.zeros(dom.domino_norm_bwd_scratch_floats(rows, h), dtype=torch.float32, device="cuda")
    md = torch.from_numpy(mean.astype(np.float32)).cuda()
    rd = torch.from_numpy(rstd.astype(np.float32)).cuda()
    dom.domino_norm_bwd(dev(ga), dev(gb), dev(x), dev(g), md, rd, dev(dres), dx, dg, None if rms else db, scratch,
                        rows, h, rms)
    torch.cuda.synchronize()
    rdx, rdg, rdb = O.norm_bwd(ga.astype(np.float64) + gb, x.astype(np.float64), g, mean, rstd, bool(rms))
    assert relerr(host(dx), rdx + dres) < 1e-2
    assert relerr(dg.cpu().numpy(), rdg) < 1e-2          # ga + gb is rounded to bf16 once before use
    if not rms:
        assert relerr(db.cpu().numpy(), rdb) < 1e-2


def _attn_inputs(rng, b, s, nh, d):
    hl = nh * d
    qkv = rnd(rng, (b * s, 3 * hl), 1.0)
    to4 = lambda m: m.reshape(b, s, nh, d).transpose(0, 2, 1, 3).astype(np.float64)
    return qkv, to4(qkv[:, :hl]), to4(qkv[:, hl:2 * hl]), to4(qkv[:, 2 * hl:])


@pytest.mark.parametrize("d", [64, 80, 128])
@pytest.mark.parametrize("b,s,nh", [(2, 200, 2), (1, 384, 3), (1, 64, 1), (1, 1, 1), (3, 9, 2), (2, 640, 5)])   # s = 1: softmax over one key; the last: 50 / 100 work items dealt over 8 XCDs
def test_attention_forward(dom, d, b, s, nh):
    rng = np.random.default_rng(d + s)
    hl = nh * d
    qkv, q, k, v = _attn_inputs(rng, b, s, nh, d)
    ctx = torch.zeros((b * s, hl), dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros((b, nh, s), dtype=torch.float32, device="cuda")
    dom.domino_attention_fwd(dev(qkv), 3 * hl, b, s, nh, d, ctx, lse)
    torch.cuda.synchronize()
    rctx, rlse = O.attention_fwd(q, k, v)
    rctx2 = rctx.transpose(0, 2, 1, 3).reshape(b * s, hl)
    assert relerr(host(ctx), rctx2) < 1e-2                # probabilities are rounded to bf16 before P V
    assert np.max(np.abs(lse.cpu().numpy() - rlse)) < 2e-3
    # position 0 sees only key 0: its output is v_0 exactly (bf16 values pass through unchanged)
    got = host(ctx).reshape(b, s, nh, d)
    np.testing.assert_allclose(got[:, 0], v[:, :, 0], atol=1e-6)


@pytest.mark.parametrize("d", [64, 80, 128])
@pytest.mark.parametrize("b,s,nh", [(2, 200, 2), (1, 384, 3), (1, 1, 1), (3, 9, 2), (2, 640, 5)])
def test_attention_backward(dom, d, b, s, nh):
    rng = np.random.default_rng(d + s + 1)
    hl = nh * d
    qkv, q, k, v = _attn_inputs(rng, b, s, nh, d)
    dctx = rnd(rng, (b * s, hl))
    ctx = torch.zeros((b * s, hl), dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros((b, nh, s), dtype=torch.float32, device="cuda")
    dqkv = torch.zeros((b * s, 3 * hl), dtype=torch.bfloat16, device="cuda")
    dot = torch.zeros((b, nh, s), dtype=torch.float32, device="cuda")
    qd = dev(qkv)
    dom.domino_attention_fwd(qd, 3 * hl, b, s, nh, d, ctx, lse)
    dom.domino_attention_bwd(qd, 3 * hl, ctx, dev(dctx), lse, dqkv, dot, b, s, nh, d)
    torch.cuda.synchronize()
    d4 = dctx.reshape(b, s, nh, d).transpose(0, 2, 1, 3).astype(np.float64)
    rdq, rdk, rdv = O.attention_bwd(d4, q, k, v)
    back = lambda m: m.transpose(0, 2, 1, 3).reshape(b * s, hl)
    got = host(dqkv)
    assert relerr(got[:, :hl], back(rdq)) < 1.5e-2
    assert relerr(got[:, hl:2 * hl], back(rdk)) < 1.5e-2
    assert relerr(got[:, 2 * hl:], back(rdv)) < 1.5e-2


@pytest.mark.parametrize("inverse", [0, 1])
def test_rope(dom, inverse):
    rng = np.random.default_rng(3)
    b, s, nh, d = 2, 96, 3, 128
    hl = nh * d
    m = rnd(rng, (b * s, 3 * hl))
    md = dev(m)
    dom.domino_rope(md, 3 * hl, b * s, s, 0, 2, nh, d, 10000.0, inverse)
    torch.cuda.synchronize()
    cos, sin = O.rope_tables(s, d, 10000.0)
    ref = m.astype(np.float64).copy()
    for blk in range(2):
        part = ref[:, blk * hl:(blk + 1) * hl].reshape(b, s, nh, d).transpose(0, 2, 1, 3)
        rot = O.rope_apply(part, cos, sin, inverse=bool(inverse))
        ref[:, blk * hl:(blk + 1) * hl] = rot.transpose(0, 2, 1, 3).reshape(b * s, hl)
    got = host(md)
    assert relerr(got, ref) < 5e-3
    np.testing.assert_array_equal(got[:, 2 * hl:], m[:, 2 * hl:])       # the v block is untouched


@pytest.mark.parametrize("tile", [0, 1, 2, 3])
@pytest.mark.parametrize("d,nh,b,s", [(128, 3, 2, 200), (64, 5, 3, 72), (128, 5, 1, 264)])
def test_gemm_rope_epilogue(dom, tile, d, nh, b, s):
    """The QKV product with the rotary embedding in its epilogue against the plain product followed by the oracle's
    rotation: q and k heads turned, v heads untouched, positions wrapping at every sequence end inside a tile."""
    rng = np.random.default_rng(100 * d + nh + tile)
    hl = nh * d
    M, N, K = b * s, 3 * hl, 136
    A, B = rnd(rng, (M, K)), rnd(rng, (K, N), 0.1)
    Cd = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    dom.domino_gemm_rope(tile, dev(A), K, dev(B), N, Cd, N, M, N, K, s, d, 2 * hl, 10000.0)
    torch.cuda.synchronize()
    ref = A.astype(np.float64) @ B.astype(np.float64)
    cos, sin = O.rope_tables(s, d, 10000.0)
    for blk in range(2):
        part = ref[:, blk * hl:(blk + 1) * hl].reshape(b, s, nh, d).transpose(0, 2, 1, 3)
        ref[:, blk * hl:(blk + 1) * hl] = O.rope_apply(part, cos, sin).transpose(0, 2, 1, 3).reshape(M, hl)
    got = host(Cd)
    for blk in range(3):
        assert relerr(got[:, blk * hl:(blk + 1) * hl], ref[:, blk * hl:(blk + 1) * hl]) < BF16_OUT, blk


def test_gemm_rope_epilogue_long_sequence(dom):
    """4096 positions: the angle recurrence of the epilogue runs over every row of a tile without drifting."""
    rng = np.random.default_rng(5)
    d, nh, s, K = 128, 2, 4096, 72
    hl = nh * d
    A, B = rnd(rng, (s, K)), rnd(rng, (K, 3 * hl), 0.1)
    Cd = torch.zeros((s, 3 * hl), dtype=torch.bfloat16, device="cuda")
    dom.domino_gemm_rope(-1, dev(A), K, dev(B), 3 * hl, Cd, 3 * hl, s, 3 * hl, K, s, d, 2 * hl, 10000.0)
    torch.cuda.synchronize()
    ref = A.astype(np.float64) @ B.astype(np.float64)
    cos, sin = O.rope_tables(s, d, 10000.0)
    for blk in range(2):
        part = ref[:, blk * hl:(blk + 1) * hl].reshape(1, s, nh, d).transpose(0, 2, 1, 3)
        ref[:, blk * hl:(blk + 1) * hl] = O.rope_apply(part, cos, sin).transpose(0, 2, 1, 3).reshape(s, hl)
    assert relerr(host(Cd), ref) < BF16_OUT


@pytest.mark.parametrize("d,b,s,nh", [(64, 2, 200, 2), (80, 1, 136, 3), (128, 2, 264, 2)])
def test_attention_backward_through_the_rotary_embedding(dom, d, b, s, nh):
    """dq, dk with respect to q, k before the rotation: the oracle's attention gradients taken through its rotation."""
    rng = np.random.default_rng(d + s + 7)
    hl = nh * d
    qkv, q, k, v = _attn_inputs(rng, b, s, nh, d)          # q, k here are the rotated vectors the kernel reads
    dctx = rnd(rng, (b * s, hl))
    ctx = torch.zeros((b * s, hl), dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros((b, nh, s), dtype=torch.float32, device="cuda")
    dqkv = torch.zeros((b * s, 3 * hl), dtype=torch.bfloat16, device="cuda")
    dot = torch.zeros((b, nh, s), dtype=torch.float32, device="cuda")
    qd = dev(qkv)
    dom.domino_attention_fwd(qd, 3 * hl, b, s, nh, d, ctx, lse)
    dom.domino_attention_bwd_rope(qd, 3 * hl, ctx, dev(dctx), lse, dqkv, dot, b, s, nh, d, 10000.0)
    torch.cuda.synchronize()
    d4 = dctx.reshape(b, s, nh, d).transpose(0, 2, 1, 3).astype(np.float64)
    rdq, rdk, rdv = O.attention_bwd(d4, q, k, v)
    cos, sin = O.rope_tables(s, d, 10000.0)
    rdq, rdk = O.rope_apply(rdq, cos, sin, inverse=True), O.rope_apply(rdk, cos, sin, inverse=True)
    back = lambda m: m.transpose(0, 2, 1, 3).reshape(b * s, hl)
    got = host(dqkv)
    assert relerr(got[:, :hl], back(rdq)) < 1.5e-2
    assert relerr(got[:, hl:2 * hl], back(rdk)) < 1.5e-2
    assert relerr(got[:, 2 * hl:], back(rdv)) < 1.5e-2


def test_colsum(dom):
    rng = np.random.default_rng(4)
    rows, n, ld = 1000, 264, 328
    g = rnd(rng, (rows, ld))
    out = torch.ones(n, dtype=torch.float32, device="cuda")
    scratch = torch.zeros(64 * n, dtype=torch.float32, device="cuda")
    dom.domino_colsum(dev(g), ld, rows, n, out, 0, scratch)
    torch.cuda.synchronize()
    ref = g[:, :n].astype(np.float64).sum(0)
    assert np.max(np.abs(out.cpu().numpy() - ref)) < 1e-3
    dom.domino_colsum(dev(g), ld, rows, n, out, 1, scratch)
    torch.cuda.synchronize()
    assert np.max(np.abs(out.cpu().numpy() - 2 * ref)) < 2e-3
