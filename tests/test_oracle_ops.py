"""Pins for the oracle's building blocks: closed forms, invariants, brute force and
PyTorch-CPU library routines (never the oracle's own formula retyped)."""
import math

import numpy as np
import pytest
import torch

from oracle import domino_oracle as O

RNG = np.random.default_rng(7)


def fd(f, x, eps=1e-6):
    return (f(x + eps) - f(x - eps)) / (2 * eps)


# ------------------------------------------------------------------ GeLU / SiLU
def test_gelu_closed_forms():
    x = np.linspace(-6, 6, 241)
    for tanh in (True, False):
        assert O.gelu(np.array([0.0]), tanh)[0] == 0.0
        np.testing.assert_allclose(O.gelu(x, tanh) - O.gelu(-x, tanh), x, atol=1e-14)
    # exact GeLU(1) = Phi(1)
    assert abs(O.gelu(np.array([1.0]), False)[0] - 0.8413447460685429) < 1e-15
    assert np.max(np.abs(O.gelu(x, True) - O.gelu(x, False))) < 1e-3
    # far tails: identity / zero
    assert abs(O.gelu(np.array([30.0]))[0] - 30.0) < 1e-12 and abs(O.gelu(np.array([-30.0]))[0]) < 1e-12


def test_gelu_matches_torch_library():
    x = RNG.standard_normal(1000) * 3
    xt = torch.tensor(x, dtype=torch.float64)
    np.testing.assert_allclose(O.gelu(x, True), torch.nn.functional.gelu(xt, approximate="tanh").numpy(), atol=1e-14)
    np.testing.assert_allclose(O.gelu(x, False), torch.nn.functional.gelu(xt).numpy(), atol=1e-14)
    np.testing.assert_allclose(O.silu(x), torch.nn.functional.silu(xt).numpy(), atol=1e-14)


def test_activation_derivatives_by_finite_differences():
    x = RNG.standard_normal(500) * 2.5
    for tanh in (True, False):
        np.testing.assert_allclose(O.gelu_grad(x, tanh), fd(lambda z: O.gelu(z, tanh), x), atol=1e-8)
    np.testing.assert_allclose(O.silu_grad(x), fd(O.silu, x), atol=1e-8)
    assert abs(O.silu(np.array([1.0]))[0] - 0.7310585786300049) < 1e-15
    assert O.silu_grad(np.array([0.0]))[0] == 0.5


# ------------------------------------------------------------------ norms
@pytest.mark.parametrize("rms", [False, True])
def test_norm_invariants(rms):
    h, eps = 96, 1e-5
    x = RNG.standard_normal((3, 5, h)) * 2 + 0.7
    y, mean, rstd = O.norm_fwd(x, np.ones(h), None if rms else np.zeros(h), eps, rms)
    if rms:
        ms = (x * x).mean(-1)
        np.testing.assert_allclose((y * y).mean(-1), ms / (ms + eps), rtol=1e-12)
        y2, _, _ = O.norm_fwd(3.5 * x, np.ones(h), None, 0.0, True)     # scale invariance at eps -> 0
        y0, _, _ = O.norm_fwd(x, np.ones(h), None, 0.0, True)
        np.testing.assert_allclose(y2, y0, atol=1e-12)
        assert np.all(mean == 0)
    else:
        var = x.var(-1)
        np.testing.assert_allclose(y.mean(-1), 0, atol=1e-13)
        np.testing.assert_allclose(y.var(-1), var / (var + eps), rtol=1e-12)
        y2, _, _ = O.norm_fwd(x + 11.0, np.ones(h), np.zeros(h), eps, False)   # shift invariance
        np.testing.assert_allclose(y2, y, atol=1e-11)
        np.testing.assert_allclose(mean, x.mean(-1), atol=1e-14)


def test_layernorm_matches_torch_library_fwd_bwd():
    h, eps = 64, 1e-5
    x = RNG.standard_normal((4, 7, h))
    g, b = RNG.standard_normal(h), RNG.standard_normal(h)
    dy = RNG.standard_normal((4, 7, h))
    xt = torch.tensor(x, requires_grad=True)
    gt, bt = torch.tensor(g, requires_grad=True), torch.tensor(b, requires_grad=True)
    yt = torch.nn.functional.layer_norm(xt, (h,), gt, bt, eps)
    yt.backward(torch.tensor(dy))
    y, mean, rstd = O.norm_fwd(x, g, b, eps, False)
    dx, dg, db = O.norm_bwd(dy, x, g, mean, rstd, False)
    np.testing.assert_allclose(y, yt.detach().numpy(), atol=1e-12)
    np.testing.assert_allclose(dx, xt.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dg, gt.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(db, bt.grad.numpy(), atol=1e-12)


def test_rmsnorm_matches_torch_library_fwd_bwd():
    h, eps = 48, 1e-5
    x = RNG.standard_normal((2, 9, h))
    g = RNG.standard_normal(h)
    dy = RNG.standard_normal((2, 9, h))
    xt, gt = torch.tensor(x, requires_grad=True), torch.tensor(g, requires_grad=True)
    yt = torch.nn.functional.rms_norm(xt, (h,), gt, eps)
    yt.backward(torch.tensor(dy))
    y, mean, rstd = O.norm_fwd(x, g, None, eps, True)
    dx, dg, db = O.norm_bwd(dy, x, g, mean, rstd, True)
    assert db is None
    np.testing.assert_allclose(y, yt.detach().numpy(), atol=1e-12)
    np.testing.assert_allclose(dx, xt.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dg, gt.grad.numpy(), atol=1e-12)


# ------------------------------------------------------------------ rotary embedding
def test_rope_properties():
    s, d = 17, 16
    cos, sin = O.rope_tables(s, d, 10000.0)
    x = RNG.standard_normal((2, 3, s, d))
    y = O.rope_apply(x, cos, sin)
    np.testing.assert_allclose(y[..., 0, :], x[..., 0, :], atol=0)            # position 0: identity
    np.testing.assert_allclose(x[..., :d // 2] ** 2 + x[..., d // 2:] ** 2,
                               y[..., :d // 2] ** 2 + y[..., d // 2:] ** 2, atol=1e-12)   # pair norms
    np.testing.assert_allclose(O.rope_apply(y, cos, sin, inverse=True), x, atol=1e-13)   # inverse = transpose
    # <R x, z> = <x, R^T z>
    z = RNG.standard_normal(x.shape)
    np.testing.assert_allclose((y * z).sum(), (x * O.rope_apply(z, cos, sin, inverse=True)).sum(), rtol=1e-12)
    # the slowest pair turns by exactly m * base^(-(d-2)/d); the fastest by m radians
    e = np.zeros((s, d)); e[:, 0] = 1.0
    r = O.rope_apply(e, cos, sin)
    np.testing.assert_allclose(r[:, 0], np.cos(np.arange(s)), atol=1e-14)
    np.testing.assert_allclose(r[:, d // 2], np.sin(np.arange(s)), atol=1e-14)
    e = np.zeros((s, d)); e[:, d // 2 - 1] = 1.0
    r = O.rope_apply(e, cos, sin)
    np.testing.assert_allclose(r[:, d - 1], np.sin(np.arange(s) * 10000.0 ** (-(d - 2) / d)), atol=1e-14)


def test_rope_scores_depend_on_relative_position_only():
    s, d, c = 12, 8, 5
    cos, sin = O.rope_tables(s + c, d, 10000.0)
    q, k = RNG.standard_normal((s, d)), RNG.standard_normal((s, d))
    a = O.rope_apply(q, cos[:s], sin[:s]) @ O.rope_apply(k, cos[:s], sin[:s]).T
    b = O.rope_apply(q, cos[c:], sin[c:]) @ O.rope_apply(k, cos[c:], sin[c:]).T
    np.testing.assert_allclose(a, b, atol=1e-12)


# ------------------------------------------------------------------ attention
def _attention_loops(q, k, v):
    """Scalar-loop definition of causal attention for one head (tiny shapes)."""
    s, d = q.shape
    out = np.zeros((s, d))
    for i in range(s):
        w = [math.exp(sum(q[i, c] * k[j, c] for c in range(d)) / math.sqrt(d)) for j in range(i + 1)]
        z = sum(w)
        for j in range(i + 1):
            for c in range(d):
                out[i, c] += w[j] / z * v[j, c]
    return out


def test_attention_brute_force_and_invariants():
    b, nh, s, d = 2, 2, 9, 4
    q, k, v = (RNG.standard_normal((b, nh, s, d)) for _ in range(3))
    ctx, lse = O.attention_fwd(q, k, v)
    for bi in range(b):
        for hi in range(nh):
            np.testing.assert_allclose(ctx[bi, hi], _attention_loops(q[bi, hi], k[bi, hi], v[bi, hi]), atol=1e-13)
    P = O.attention_probs(q, k)
    np.testing.assert_allclose(P.sum(-1), 1.0, atol=1e-14)
    assert np.all(np.triu(P[0, 0], 1) == 0)
    np.testing.assert_allclose(ctx[:, :, 0], v[:, :, 0], atol=1e-14)            # one unmasked key
    # log-sum-exp against its definition on the unmasked scores
    sc = np.einsum("bhid,bhjd->bhij", q, k) / math.sqrt(d)
    for i in range(s):
        np.testing.assert_allclose(lse[..., i], np.log(np.exp(sc[..., i, :i + 1]).sum(-1)), atol=1e-13)
    # batch permutation commutes (row slicing relies on it)
    ctx_p, _ = O.attention_fwd(q[::-1], k[::-1], v[::-1])
    np.testing.assert_allclose(ctx_p, ctx[::-1], atol=0)
    # future tokens never reach the past
    k2, v2 = k.copy(), v.copy()
    k2[:, :, 5:] += 3.0; v2[:, :, 5:] -= 2.0
    ctx2, _ = O.attention_fwd(q, k2, v2)
    np.testing.assert_allclose(ctx2[:, :, :5], ctx[:, :, :5], atol=0)


def test_attention_equal_keys_gives_running_mean():
    s, d = 11, 6
    q = RNG.standard_normal((1, 1, s, d))
    k = np.tile(RNG.standard_normal((1, 1, 1, d)), (1, 1, s, 1))
    v = RNG.standard_normal((1, 1, s, d))
    ctx, _ = O.attention_fwd(q, k, v)
    np.testing.assert_allclose(ctx[0, 0], np.cumsum(v[0, 0], 0) / np.arange(1, s + 1)[:, None], atol=1e-13)


def test_attention_matches_torch_sdpa_fwd_bwd():
    b, nh, s, d = 2, 3, 16, 8
    q, k, v, do = (RNG.standard_normal((b, nh, s, d)) for _ in range(4))
    qt, kt, vt = (torch.tensor(a, requires_grad=True) for a in (q, k, v))
    ot = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, is_causal=True)
    ot.backward(torch.tensor(do))
    ctx, _ = O.attention_fwd(q, k, v)
    dq, dk, dv = O.attention_bwd(do, q, k, v)
    np.testing.assert_allclose(ctx, ot.detach().numpy(), atol=1e-12)
    np.testing.assert_allclose(dq, qt.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dk, kt.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dv, vt.grad.numpy(), atol=1e-12)
