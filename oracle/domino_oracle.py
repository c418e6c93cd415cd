"""CPU oracle for one tensor-parallel rank's transformer layer, Domino-sliced.

TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64 NumPy written from the paper's
definitions; it shares no code with the HIP library and must never be reached
from the product path.  Only tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import it.

What it computes (paper passages, by section / equation):
  * Sec. 3.1, Eq. 1: a sub-layer is  X (x) A (x) B = Y.  Tensor parallelism cuts
    A by columns and B by rows over t ranks; the rank outputs Y_r sum to Y.
  * Sec. 3.2, Eq. 2: X (x) A is softmax(QK^T/sqrt(d_k)) V for attention and a plain
    product for the MLP; Eq. 3: cutting X along the batch dimension leaves every
    output row unchanged.
  * Sec. 3.3, Eq. 4: cutting B by columns yields column blocks of Y that are
    concatenated; Sec. 3.4: both cuts together give a p x q grid of pieces.
  * Sec. 2.3 (Fig. 2): a block is self-attention then MLP, with one all-reduce
    after each in forward and one before each in backward.
  * Sec. 4.1 lists the ops around the products: LayerNorm, residual, dropout,
    GeLU; Sec. 5.4: Llama-2 replaces them with RMSNorm, SwiGLU and rotary
    embedding.
Readings where the paper is silent (pre-norm block, causal mask, no dropout,
tanh GeLU by default, eps inside the square root, biases of the row-cut products
added once after the reduction, rotate-half rotary pairing) are listed in the
repository's design notes.

Every public function is pinned by a non-GPU test against something other than
itself: closed forms, invariants, brute-force loops, finite differences, and a
PyTorch-CPU autograd composition.  No function here is "parity unpinned".

Conventions: all arrays float64; activations [b, s, h]; matrices row-major
[in, out]; a params dict uses the twelve names norm1_g, norm1_b, w_qkv, b_qkv,
w_o, b_o, norm2_g, norm2_b, w_up, b_up, w_down, b_down (None where the
architecture has no such tensor).  ``cfg`` is any object with attributes hidden,
heads, tp, rank, p, q, batch, seq, ffn, arch (0 GPT, 1 Llama), gelu_tanh,
norm_eps, rope_base.
"""
from __future__ import annotations

import math
from types import SimpleNamespace

import numpy as np

GPT, LLAMA = 0, 1
_F = np.float64


# --------------------------------------------------------------------------- helpers
def _f(a):
    return None if a is None else np.asarray(a, dtype=_F)


def _dims(cfg):
    h, n, t = cfg.hidden, cfg.heads, cfg.tp
    d = h // n
    nl = n // t
    return SimpleNamespace(h=h, n=n, t=t, d=d, nl=nl, hl=nl * d, fl=cfg.ffn // t,
                           b=cfg.batch, s=cfg.seq)


def check_divisible(cfg):
    """The cuts must be exact: batch by p (Sec. 4.1.1), hidden by q (Sec. 4.2), heads and ffn by t."""
    ok = (cfg.hidden % cfg.heads == 0 and cfg.heads % cfg.tp == 0 and cfg.ffn % cfg.tp == 0
          and cfg.batch % cfg.p == 0 and cfg.hidden % cfg.q == 0 and 0 <= cfg.rank < cfg.tp)
    if not ok:
        raise ValueError("configuration does not divide evenly")


# --------------------------------------------------------------------------- element-wise ops
_K0 = math.sqrt(2.0 / math.pi)
_K1 = 0.044715


def _erf(x):
    from scipy.special import erf  # library primitive used as one step
    return erf(x)


def gelu(x, tanh_approx=True):
    x = _f(x)
    if tanh_approx:
        return 0.5 * x * (1.0 + np.tanh(_K0 * (x + _K1 * x ** 3)))
    return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0)))


def gelu_grad(x, tanh_approx=True):
    x = _f(x)
    if tanh_approx:
        th = np.tanh(_K0 * (x + _K1 * x ** 3))
        return 0.5 * (1.0 + th) + 0.5 * x * (1.0 - th * th) * _K0 * (1.0 + 3.0 * _K1 * x * x)
    cdf = 0.5 * (1.0 + _erf(x / math.sqrt(2.0)))
    pdf = np.exp(-0.5 * x * x) / math.sqrt(2.0 * math.pi)
    return cdf + x * pdf


def sigmoid(x):
    x = _f(x)
    out = np.empty_like(x)
    pos = x >= 0
    out[pos] = 1.0 / (1.0 + np.exp(-x[pos]))
    e = np.exp(x[~pos])
    out[~pos] = e / (1.0 + e)
    return out


def silu(x):
    return _f(x) * sigmoid(x)


def silu_grad(x):
    sg = sigmoid(x)
    return sg * (1.0 + _f(x) * (1.0 - sg))


# --------------------------------------------------------------------------- normalisation
def norm_fwd(x, g, b, eps, rms):
    """LayerNorm (rms=False) or RMSNorm (rms=True) over the last axis.

    Returns y and the per-row statistics (mean, rstd); mean is 0 for RMSNorm."""
    x = _f(x)
    if rms:
        mean = np.zeros(x.shape[:-1], dtype=_F)
        rstd = 1.0 / np.sqrt((x * x).mean(axis=-1) + eps)
    else:
        mean = x.mean(axis=-1)
        var = ((x - mean[..., None]) ** 2).mean(axis=-1)
        rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mean[..., None]) * rstd[..., None]
    y = xhat * _f(g)
    if b is not None:
        y = y + _f(b)
    return y, mean, rstd


def norm_bwd(dy, x, g, mean, rstd, rms):
    """Gradients of norm_fwd: dx, dg, db (db is None for RMSNorm)."""
    dy, x = _f(dy), _f(x)
    xhat = (x - mean[..., None]) * rstd[..., None]
    dxhat = dy * _f(g)
    c2 = (dxhat * xhat).mean(axis=-1, keepdims=True)
    if rms:
        dx = rstd[..., None] * (dxhat - xhat * c2)
        db = None
    else:
        c1 = dxhat.mean(axis=-1, keepdims=True)
        dx = rstd[..., None] * (dxhat - c1 - xhat * c2)
        db = dy.reshape(-1, dy.shape[-1]).sum(axis=0)
    dg = (dy * xhat).reshape(-1, dy.shape[-1]).sum(axis=0)
    return dx, dg, db


# --------------------------------------------------------------------------- rotary embedding
def rope_tables(seq, d, base):
    """cos/sin [seq, d/2] for positions 0..seq-1 and frequencies base^(-2i/d)."""
    i = np.arange(d // 2, dtype=_F)
    freq = base ** (-2.0 * i / d)
    ang = np.arange(seq, dtype=_F)[:, None] * freq[None, :]
    return np.cos(ang), np.sin(ang)


def rope_apply(x, cos, sin, inverse=False):
    """Rotate pairs (i, i + d/2) of x [..., s, d] by the position angle (its transpose if inverse)."""
    x = _f(x)
    half = x.shape[-1] // 2
    x1, x2 = x[..., :half], x[..., half:]
    if inverse:
        sin = -sin
    return np.concatenate([x1 * cos - x2 * sin, x2 * cos + x1 * sin], axis=-1)


# --------------------------------------------------------------------------- attention (Eq. 2, first case)
def attention_fwd(q, k, v):
    """Causal softmax(q k^T / sqrt(d)) v for q, k, v of shape [b, heads, s, d].

    Returns ctx [b, heads, s, d] and the log-sum-exp of the scaled, masked scores [b, heads, s]."""
    q, k, v = _f(q), _f(k), _f(v)
    b, nh, s, d = q.shape
    ctx = np.empty_like(q)
    lse = np.empty((b, nh, s), dtype=_F)
    keep = np.tril(np.ones((s, s), dtype=bool))
    scale = 1.0 / math.sqrt(d)
    for bi in range(b):
        for hi in range(nh):
            sc = (q[bi, hi] @ k[bi, hi].T) * scale
            sc = np.where(keep, sc, -np.inf)
            m = sc.max(axis=-1, keepdims=True)
            e = np.exp(sc - m)
            z = e.sum(axis=-1, keepdims=True)
            ctx[bi, hi] = (e / z) @ v[bi, hi]
            lse[bi, hi] = (m + np.log(z))[:, 0]
    return ctx, lse


def attention_probs(q, k):
    """The probability matrix itself, [b, heads, s, s] (tests only; small shapes)."""
    q, k = _f(q), _f(k)
    s, d = q.shape[-2], q.shape[-1]
    sc = np.einsum("bhid,bhjd->bhij", q, k) / math.sqrt(d)
    sc = np.where(np.tril(np.ones((s, s), dtype=bool)), sc, -np.inf)
    e = np.exp(sc - sc.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def attention_bwd(dctx, q, k, v):
    """Gradients of attention_fwd w.r.t. q, k, v."""
    dctx, q, k, v = _f(dctx), _f(q), _f(k), _f(v)
    b, nh, s, d = q.shape
    dq, dk, dv = np.empty_like(q), np.empty_like(k), np.empty_like(v)
    keep = np.tril(np.ones((s, s), dtype=bool))
    scale = 1.0 / math.sqrt(d)
    for bi in range(b):
        for hi in range(nh):
            sc = (q[bi, hi] @ k[bi, hi].T) * scale
            sc = np.where(keep, sc, -np.inf)
            e = np.exp(sc - sc.max(axis=-1, keepdims=True))
            P = e / e.sum(axis=-1, keepdims=True)
            dP = dctx[bi, hi] @ v[bi, hi].T
            dv[bi, hi] = P.T @ dctx[bi, hi]
            dS = P * (dP - (dP * P).sum(axis=-1, keepdims=True))
            dq[bi, hi] = (dS @ k[bi, hi]) * scale
            dk[bi, hi] = (dS.T @ q[bi, hi]) * scale
    return dq, dk, dv


# --------------------------------------------------------------------------- sharding bookkeeping (Sec. 3.1)
def shard_params(full, cfg, r):
    """Rank r's share of full-width parameters: A-type matrices by columns, B-type by rows."""
    D = _dims(cfg)
    h, hl, fl = D.h, D.hl, D.fl
    P = {}
    wq = _f(full["w_qkv"])                                   # [h, 3h] = [Q | K | V]
    cols = np.concatenate([np.arange(r * hl, (r + 1) * hl) + blk * h for blk in range(3)])
    P["w_qkv"] = wq[:, cols]
    P["b_qkv"] = None if full.get("b_qkv") is None else _f(full["b_qkv"])[cols]
    P["w_o"] = _f(full["w_o"])[r * hl:(r + 1) * hl, :]
    wu = _f(full["w_up"])
    if cfg.arch == LLAMA:                                    # [h, 2f] = [gate | up]
        f = cfg.ffn
        ucols = np.concatenate([np.arange(r * fl, (r + 1) * fl), np.arange(r * fl, (r + 1) * fl) + f])
    else:
        ucols = np.arange(r * fl, (r + 1) * fl)
    P["w_up"] = wu[:, ucols]
    P["b_up"] = None if full.get("b_up") is None else _f(full["b_up"])[ucols]
    P["w_down"] = _f(full["w_down"])[r * fl:(r + 1) * fl, :]
    for kname in ("norm1_g", "norm1_b", "b_o", "norm2_g", "norm2_b", "b_down"):
        P[kname] = _f(full.get(kname))
    return P


def full_from_shards(shards, cfg):
    """Inverse of shard_params: glue the t rank shards back into full-width parameters."""
    D = _dims(cfg)
    hl, fl = D.hl, D.fl
    full = {}
    full["w_qkv"] = np.concatenate([_f(s["w_qkv"])[:, blk * hl:(blk + 1) * hl]
                                    for blk in range(3) for s in shards], axis=1)
    full["b_qkv"] = None if shards[0]["b_qkv"] is None else np.concatenate(
        [_f(s["b_qkv"])[blk * hl:(blk + 1) * hl] for blk in range(3) for s in shards])
    full["w_o"] = np.concatenate([_f(s["w_o"]) for s in shards], axis=0)
    if cfg.arch == LLAMA:
        full["w_up"] = np.concatenate([_f(s["w_up"])[:, blk * fl:(blk + 1) * fl]
                                       for blk in range(2) for s in shards], axis=1)
        full["b_up"] = None
    else:
        full["w_up"] = np.concatenate([_f(s["w_up"]) for s in shards], axis=1)
        full["b_up"] = None if shards[0]["b_up"] is None else np.concatenate([_f(s["b_up"]) for s in shards])
    full["w_down"] = np.concatenate([_f(s["w_down"]) for s in shards], axis=0)
    for kname in ("norm1_g", "norm1_b", "b_o", "norm2_g", "norm2_b", "b_down"):
        full[kname] = _f(shards[0][kname])
    return full


# --------------------------------------------------------------------------- one rank, unsliced
def _split_heads(m2, b, s, nh, d):
    return m2.reshape(b, s, nh, d).transpose(0, 2, 1, 3)


def _merge_heads(m4):
    b, nh, s, d = m4.shape
    return m4.transpose(0, 2, 1, 3).reshape(b, s, nh * d)


def rank_layer_fwd(cfg, P, x, attn_others=None, mlp_others=None):
    """Forward of one rank's share of the block on x [b, s, h] (any b).

    attn_partial = (X (x) A_r (x) B_r) of the attention sub-layer, mlp_partial likewise for
    the MLP: the tensors the two forward all-reduces would sum.  ``*_others`` stand for the sum
    of the other ranks' partials (None = zero).  Returns a dict with the partials, y and every
    intermediate the backward needs."""
    x = _f(x)
    b, s, h = x.shape
    n_local = P["w_qkv"].shape[1] // 3 // (cfg.hidden // cfg.heads)
    d = cfg.hidden // cfg.heads
    hl = n_local * d
    rms = cfg.arch == LLAMA
    ao = 0.0 if attn_others is None else _f(attn_others)
    mo = 0.0 if mlp_others is None else _f(mlp_others)

    ln1, mean1, rstd1 = norm_fwd(x, P["norm1_g"], P["norm1_b"], cfg.norm_eps, rms)
    qkv = ln1 @ _f(P["w_qkv"])
    if P["b_qkv"] is not None:
        qkv = qkv + _f(P["b_qkv"])
    q = _split_heads(qkv[..., 0 * hl:1 * hl], b, s, n_local, d)
    k = _split_heads(qkv[..., 1 * hl:2 * hl], b, s, n_local, d)
    v = _split_heads(qkv[..., 2 * hl:3 * hl], b, s, n_local, d)
    if rms:
        cos, sin = rope_tables(s, d, cfg.rope_base)
        q, k = rope_apply(q, cos, sin), rope_apply(k, cos, sin)
    ctx4, lse = attention_fwd(q, k, v)
    ctx = _merge_heads(ctx4)
    attn_partial = ctx @ _f(P["w_o"])
    x1 = x + attn_partial + ao
    if P["b_o"] is not None:
        x1 = x1 + _f(P["b_o"])
    ln2, mean2, rstd2 = norm_fwd(x1, P["norm2_g"], P["norm2_b"], cfg.norm_eps, rms)
    pre = ln2 @ _f(P["w_up"])
    if P["b_up"] is not None:
        pre = pre + _f(P["b_up"])
    if rms:
        fl = pre.shape[-1] // 2
        act = silu(pre[..., :fl]) * pre[..., fl:]
    else:
        act = gelu(pre, bool(cfg.gelu_tanh))
    mlp_partial = act @ _f(P["w_down"])
    y = x1 + mlp_partial + mo
    if P["b_down"] is not None:
        y = y + _f(P["b_down"])
    return dict(x=x, ln1=ln1, mean1=mean1, rstd1=rstd1, q=q, k=k, v=v, lse=lse, ctx=ctx,
                attn_partial=attn_partial, x1=x1, ln2=ln2, mean2=mean2, rstd2=rstd2,
                pre=pre, act=act, mlp_partial=mlp_partial, y=y)


def rank_layer_bwd(cfg, P, S, dy, dln2_others=None, dln1_others=None):
    """Backward of rank_layer_fwd for L = sum(y * dy); S is the dict the forward returned.

    dln2_partial / dln1_partial are this rank's input-gradients of the two column-cut
    products: what the two backward all-reduces would sum.  ``dln*_others`` stand for the
    other ranks' sums.  Returns dx, the two partials and the twelve parameter gradients."""
    dy = _f(dy)
    b, s, h = dy.shape
    rms = cfg.arch == LLAMA
    d = cfg.hidden // cfg.heads
    hl = S["ctx"].shape[-1]
    n_local = hl // d
    G = {}
    flat = lambda a: a.reshape(-1, a.shape[-1])

    # MLP: y = x1 + act @ w_down + b_down (+ others)
    G["b_down"] = None if P["b_down"] is None else flat(dy).sum(axis=0)
    d_act = dy @ _f(P["w_down"]).T
    G["w_down"] = flat(S["act"]).T @ flat(dy)
    pre = S["pre"]
    if rms:
        fl = pre.shape[-1] // 2
        g_, u_ = pre[..., :fl], pre[..., fl:]
        d_pre = np.concatenate([d_act * u_ * silu_grad(g_), d_act * silu(g_)], axis=-1)
    else:
        d_pre = d_act * gelu_grad(pre, bool(cfg.gelu_tanh))
    G["w_up"] = flat(S["ln2"]).T @ flat(d_pre)
    G["b_up"] = None if P["b_up"] is None else flat(d_pre).sum(axis=0)
    dln2_partial = d_pre @ _f(P["w_up"]).T
    dln2 = dln2_partial + (0.0 if dln2_others is None else _f(dln2_others))
    dx1_n, G["norm2_g"], db2 = norm_bwd(dln2, S["x1"], P["norm2_g"], S["mean2"], S["rstd2"], rms)
    G["norm2_b"] = None if P["norm2_b"] is None else db2
    dx1 = dy + dx1_n

    # attention: x1 = x + ctx @ w_o + b_o (+ others)
    G["b_o"] = None if P["b_o"] is None else flat(dx1).sum(axis=0)
    dctx = dx1 @ _f(P["w_o"]).T
    G["w_o"] = flat(S["ctx"]).T @ flat(dx1)
    dq, dk, dv = attention_bwd(_split_heads(dctx, b, s, n_local, d), S["q"], S["k"], S["v"])
    if rms:
        cos, sin = rope_tables(s, d, cfg.rope_base)
        dq, dk = rope_apply(dq, cos, sin, inverse=True), rope_apply(dk, cos, sin, inverse=True)
    dqkv = np.concatenate([_merge_heads(dq), _merge_heads(dk), _merge_heads(dv)], axis=-1)
    G["w_qkv"] = flat(S["ln1"]).T @ flat(dqkv)
    G["b_qkv"] = None if P["b_qkv"] is None else flat(dqkv).sum(axis=0)
    dln1_partial = dqkv @ _f(P["w_qkv"]).T
    dln1 = dln1_partial + (0.0 if dln1_others is None else _f(dln1_others))
    dx_n, G["norm1_g"], db1 = norm_bwd(dln1, S["x"], P["norm1_g"], S["mean1"], S["rstd1"], rms)
    G["norm1_b"] = None if P["norm1_b"] is None else db1
    dx = dx1 + dx_n
    return dict(dx=dx, dx1=dx1, dln2_partial=dln2_partial, dln1_partial=dln1_partial,
                d_pre=d_pre, dctx=dctx, dqkv=dqkv, grads=G)


# --------------------------------------------------------------------------- the Domino p x q grid
def _col_slices(h, q):
    w = h // q
    return [slice(j * w, (j + 1) * w) for j in range(q)]


def _row_slices(b, p):
    w = b // p
    return [slice(i * w, (i + 1) * w) for i in range(p)]


def domino_layer_fwd(cfg, P, x, attn_others=None, mlp_others=None):
    """The rank's forward done piece by piece (Sec. 3.4): p row slices of the batch, and for
    the second product of each sub-layer q column slices of B whose outputs are written side
    by side (Eq. 4).  Returns the same dict layout as rank_layer_fwd plus 'pieces', a list of
    per-row-slice dicts."""
    check_divisible(cfg)
    x = _f(x)
    b, s, h = x.shape
    rms = cfg.arch == LLAMA
    cs = _col_slices(h, cfg.q)
    pieces = []
    for rs in _row_slices(b, cfg.p):
        xi = x[rs]
        ao = None if attn_others is None else _f(attn_others)[rs]
        mo = None if mlp_others is None else _f(mlp_others)[rs]
        # X (x) A: never column-sliced (Sec. 3.1, last paragraph but one)
        Pa = dict(P)
        head = rank_layer_fwd_attention_A(cfg, Pa, xi)
        attn_partial = np.empty_like(xi)
        for cj in cs:                                    # (XA) (x) B_j, Eq. 4
            attn_partial[..., cj] = head["ctx"] @ _f(P["w_o"])[:, cj]
        x1 = xi + attn_partial + (0.0 if ao is None else ao)   # needs all q column pieces
        if P["b_o"] is not None:
            x1 = x1 + _f(P["b_o"])
        ln2, mean2, rstd2 = norm_fwd(x1, P["norm2_g"], P["norm2_b"], cfg.norm_eps, rms)
        pre = ln2 @ _f(P["w_up"])
        if P["b_up"] is not None:
            pre = pre + _f(P["b_up"])
        if rms:
            fl = pre.shape[-1] // 2
            act = silu(pre[..., :fl]) * pre[..., fl:]
        else:
            act = gelu(pre, bool(cfg.gelu_tanh))
        mlp_partial = np.empty_like(xi)
        for cj in cs:
            mlp_partial[..., cj] = act @ _f(P["w_down"])[:, cj]
        y = x1 + mlp_partial + (0.0 if mo is None else mo)
        if P["b_down"] is not None:
            y = y + _f(P["b_down"])
        head.update(attn_partial=attn_partial, x1=x1, ln2=ln2, mean2=mean2, rstd2=rstd2,
                    pre=pre, act=act, mlp_partial=mlp_partial, y=y)
        pieces.append(head)
    out = {kname: np.concatenate([pc[kname] for pc in pieces], axis=0) for kname in pieces[0]}
    out["pieces"] = pieces
    return out


def rank_layer_fwd_attention_A(cfg, P, x):
    """X (x) A of the attention sub-layer for one row slice: norm, QKV product, (rotary), attention."""
    b, s, h = x.shape
    d = cfg.hidden // cfg.heads
    hl = P["w_qkv"].shape[1] // 3
    n_local = hl // d
    rms = cfg.arch == LLAMA
    ln1, mean1, rstd1 = norm_fwd(x, P["norm1_g"], P["norm1_b"], cfg.norm_eps, rms)
    qkv = ln1 @ _f(P["w_qkv"])
    if P["b_qkv"] is not None:
        qkv = qkv + _f(P["b_qkv"])
    q = _split_heads(qkv[..., :hl], b, s, n_local, d)
    k = _split_heads(qkv[..., hl:2 * hl], b, s, n_local, d)
    v = _split_heads(qkv[..., 2 * hl:], b, s, n_local, d)
    if rms:
        cos, sin = rope_tables(s, d, cfg.rope_base)
        q, k = rope_apply(q, cos, sin), rope_apply(k, cos, sin)
    ctx4, lse = attention_fwd(q, k, v)
    return dict(x=x, ln1=ln1, mean1=mean1, rstd1=rstd1, q=q, k=k, v=v, lse=lse, ctx=_merge_heads(ctx4))


def domino_layer_bwd(cfg, P, S, dy, dln2_others=None, dln1_others=None):
    """The rank's backward piece by piece: per row slice the input-gradient of each product is
    formed before its weight-gradient (Sec. 4.1.2); contributions of the q column slices of B
    are summed into the gradient of (XA); weight gradients are summed over the p row slices."""
    check_divisible(cfg)
    dy = _f(dy)
    b, s, h = dy.shape
    rms = cfg.arch == LLAMA
    d = cfg.hidden // cfg.heads
    cs = _col_slices(h, cfg.q)
    flat = lambda a: a.reshape(-1, a.shape[-1])
    G = {kname: None for kname in P}
    outs = []

    def acc(name, val):
        if P[name] is None:
            return
        G[name] = val if G[name] is None else G[name] + val

    for i, rs in enumerate(_row_slices(b, cfg.p)):
        Si = S["pieces"][i]
        dyi = dy[rs]
        hl = Si["ctx"].shape[-1]
        n_local = hl // d
        bi = dyi.shape[0]
        acc("b_down", flat(dyi).sum(axis=0))
        d_act = np.zeros_like(Si["act"])
        gw_down = np.empty_like(_f(P["w_down"]))
        for cj in cs:
            d_act += dyi[..., cj] @ _f(P["w_down"])[:, cj].T           # input-gradient first
        for cj in cs:
            gw_down[:, cj] = flat(Si["act"]).T @ flat(dyi[..., cj])
        acc("w_down", gw_down)
        pre = Si["pre"]
        if rms:
            fl = pre.shape[-1] // 2
            g_, u_ = pre[..., :fl], pre[..., fl:]
            d_pre = np.concatenate([d_act * u_ * silu_grad(g_), d_act * silu(g_)], axis=-1)
        else:
            d_pre = d_act * gelu_grad(pre, bool(cfg.gelu_tanh))
        dln2_partial = d_pre @ _f(P["w_up"]).T
        acc("w_up", flat(Si["ln2"]).T @ flat(d_pre))
        acc("b_up", flat(d_pre).sum(axis=0))
        dln2 = dln2_partial + (0.0 if dln2_others is None else _f(dln2_others)[rs])
        dx1_n, dg2, db2 = norm_bwd(dln2, Si["x1"], P["norm2_g"], Si["mean2"], Si["rstd2"], rms)
        acc("norm2_g", dg2)
        acc("norm2_b", db2)
        dx1 = dyi + dx1_n
        acc("b_o", flat(dx1).sum(axis=0))
        dctx = np.zeros_like(Si["ctx"])
        gw_o = np.empty_like(_f(P["w_o"]))
        for cj in cs:
            dctx += dx1[..., cj] @ _f(P["w_o"])[:, cj].T
        for cj in cs:
            gw_o[:, cj] = flat(Si["ctx"]).T @ flat(dx1[..., cj])
        acc("w_o", gw_o)
        dq, dk, dv = attention_bwd(_split_heads(dctx, bi, s, n_local, d), Si["q"], Si["k"], Si["v"])
        if rms:
            cos, sin = rope_tables(s, d, cfg.rope_base)
            dq, dk = rope_apply(dq, cos, sin, inverse=True), rope_apply(dk, cos, sin, inverse=True)
        dqkv = np.concatenate([_merge_heads(dq), _merge_heads(dk), _merge_heads(dv)], axis=-1)
        dln1_partial = dqkv @ _f(P["w_qkv"]).T
        acc("w_qkv", flat(Si["ln1"]).T @ flat(dqkv))
        acc("b_qkv", flat(dqkv).sum(axis=0))
        dln1 = dln1_partial + (0.0 if dln1_others is None else _f(dln1_others)[rs])
        dx_n, dg1, db1 = norm_bwd(dln1, Si["x"], P["norm1_g"], Si["mean1"], Si["rstd1"], rms)
        acc("norm1_g", dg1)
        acc("norm1_b", db1)
        outs.append(dict(dx=dx1 + dx_n, dx1=dx1, dln2_partial=dln2_partial, dln1_partial=dln1_partial,
                         d_pre=d_pre, dctx=dctx, dqkv=dqkv))
    out = {kname: np.concatenate([o[kname] for o in outs], axis=0) for kname in outs[0]}
    out["grads"] = G
    return out


# --------------------------------------------------------------------------- all ranks / no sharding
def full_layer_fwd(cfg, full, x):
    """The unsharded, unsliced block (t = p = q = 1) on full-width parameters."""
    one = SimpleNamespace(**{**_cfg_dict(cfg), "tp": 1, "rank": 0, "p": 1, "q": 1})
    return rank_layer_fwd(one, {kname: _f(v) for kname, v in full.items()}, x)


def full_layer_bwd(cfg, full, S, dy):
    one = SimpleNamespace(**{**_cfg_dict(cfg), "tp": 1, "rank": 0, "p": 1, "q": 1})
    return rank_layer_bwd(one, {kname: _f(v) for kname, v in full.items()}, S, dy)


def _cfg_dict(cfg):
    return {a: getattr(cfg, a) for a in ("hidden", "heads", "tp", "rank", "p", "q", "batch", "seq",
                                         "ffn", "arch", "gelu_tanh", "norm_eps", "rope_base")}


def simulate_tp(cfg, shards, x, dy):
    """Run all t ranks and perform the four all-reduces of a block (Sec. 2.3) as plain sums.

    Because x1 of every rank depends on the reduced attention output, the forward goes in two
    phases.  Returns per-rank forward/backward dicts (each rank's y equals the full layer's)."""
    t = cfg.tp
    x, dy = _f(x), _f(dy)
    first = [rank_layer_fwd(cfg, shards[r], x) for r in range(t)]
    attn = [f["attn_partial"] for f in first]
    attn_sum = sum(attn)
    second = [rank_layer_fwd(cfg, shards[r], x, attn_others=attn_sum - attn[r]) for r in range(t)]
    mlp = [f["mlp_partial"] for f in second]
    mlp_sum = sum(mlp)
    fwd = [rank_layer_fwd(cfg, shards[r], x, attn_others=attn_sum - attn[r], mlp_others=mlp_sum - mlp[r])
           for r in range(t)]
    b1 = [rank_layer_bwd(cfg, shards[r], fwd[r], dy) for r in range(t)]
    d2 = [o["dln2_partial"] for o in b1]
    d2_sum = sum(d2)
    b2 = [rank_layer_bwd(cfg, shards[r], fwd[r], dy, dln2_others=d2_sum - d2[r]) for r in range(t)]
    d1 = [o["dln1_partial"] for o in b2]
    d1_sum = sum(d1)
    bwd = [rank_layer_bwd(cfg, shards[r], fwd[r], dy, dln2_others=d2_sum - d2[r],
                          dln1_others=d1_sum - d1[r]) for r in range(t)]
    return fwd, bwd


# --------------------------------------------------------------------------- a stack of blocks
def rank_stack_fwd(cfg, Ps, x, others=None):
    """N blocks one after the other (Sec. 2.3): block l's input is block l-1's output y.

    Ps is a list of parameter dicts; ``others`` an optional list of dicts with attn_others /
    mlp_others per block.  Returns the list of per-block forward dicts (the last one's 'y' is
    the stack's output)."""
    outs = []
    cur = _f(x)
    for l, P in enumerate(Ps):
        o = {} if others is None else others[l]
        S = rank_layer_fwd(cfg, P, cur, o.get("attn_others"), o.get("mlp_others"))
        outs.append(S)
        cur = S["y"]
    return outs


def rank_stack_bwd(cfg, Ps, Ss, dy, others=None):
    """Backward of rank_stack_fwd for L = sum(y_last * dy): the blocks in reverse, dx of block l
    being dy of block l-1.  Returns the list of per-block backward dicts in block order (the
    first one's 'dx' is the gradient of the stack's input)."""
    outs = [None] * len(Ps)
    cur = _f(dy)
    for l in reversed(range(len(Ps))):
        o = {} if others is None else others[l]
        outs[l] = rank_layer_bwd(cfg, Ps[l], Ss[l], cur, o.get("dln2_others"), o.get("dln1_others"))
        cur = outs[l]["dx"]
    return outs


# --------------------------------------------------------------------------- flop bookkeeping
def algorithmic_flops(cfg):
    """Forward+backward matmul flops of one rank's layer: causal attention counted at half the
    dense s^2, backward = 2 x forward, recomputation not counted."""
    D = _dims(cfg)
    M = D.b * D.s
    u = D.fl * (2 if cfg.arch == LLAMA else 1)
    gemm = 2.0 * M * (D.h * 3 * D.hl + D.hl * D.h + D.h * u + D.fl * D.h)
    attn = 2.0 * D.b * D.nl * D.s * D.s * D.d
    return 3.0 * (gemm + attn)
