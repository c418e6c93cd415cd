"""Seeded synthetic inputs for one tensor-parallel rank's transformer-layer shard.

This module only draws random numbers and rounds them to bf16; it holds none of
the layer's arithmetic.  Both the CPU oracle's tests and the HIP path's tests /
benchmark take their inputs from here so that they see identical values.

Shapes follow the workloads of the paper's evaluation (GPT-3 and Llama-2 model
families, Table 1 and Sec. 5.1) cut the Megatron way (Sec. 3.1: first weight
group by columns, second by rows).  Values: activations and incoming gradients
~ N(0,1); weight matrices ~ N(0, 0.02^2); norm gains 1, norm shifts and biases 0
unless ``random_affine`` is set.  Everything is rounded to bf16
(round-to-nearest-even) and handed out as float32 arrays holding exactly
representable bf16 values.

Every rank's weight shard comes from its own counter-free PCG64 stream keyed by
(seed, tensor id, rank), so the full-width matrix is by construction the
concatenation of the t rank shards and a large configuration never has to
materialise the ranks it does not use.
"""
from __future__ import annotations

import dataclasses
from typing import Dict

import numpy as np

ARCH_GPT = 0    # LayerNorm, biases, GeLU
ARCH_LLAMA = 1  # RMSNorm, no biases, SwiGLU, rotary embedding on q and k

BASE_SEED = 20240915


@dataclasses.dataclass(frozen=True)
class ShardConfig:
    """Scalars that name one rank's shard and its Domino slicing.

    hidden h, heads n, tp t, rank r, row slices p (the paper's p1, Sec. 4.1),
    column slices q (the paper's p2, Sec. 4.2), batch b, seq s, ffn f (full width).
    """
    name: str
    hidden: int
    heads: int
    tp: int
    rank: int
    p: int
    q: int
    batch: int
    seq: int
    ffn: int
    arch: int = ARCH_GPT
    gelu_tanh: int = 1
    norm_eps: float = 1e-5
    rope_base: float = 10000.0
    index: int = 0          # position in the workload table: offsets the seed
    wgrad_per_slice: int = 0    # 1: weight gradients slice by slice also for p > 2 (the order of Sec. 4.1.2)

    @property
    def head_dim(self) -> int:
        return self.hidden // self.heads

    @property
    def local_heads(self) -> int:
        return self.heads // self.tp

    @property
    def h_local(self) -> int:
        return self.local_heads * self.head_dim

    @property
    def f_local(self) -> int:
        return self.ffn // self.tp

    @property
    def up_cols(self) -> int:
        return self.f_local * (2 if self.arch == ARCH_LLAMA else 1)

    @property
    def tokens(self) -> int:
        return self.batch * self.seq

    def replace(self, **kw) -> "ShardConfig":
        return dataclasses.replace(self, **kw)


WORKLOADS: Dict[str, ShardConfig] = {
    "tiny": ShardConfig("tiny", 256, 4, 2, 0, 2, 2, 2, 128, 1024, ARCH_GPT, index=0),
    "gpt3-2.7b": ShardConfig("gpt3-2.7b", 2560, 32, 8, 0, 2, 2, 8, 2048, 10240, ARCH_GPT, index=1),
    "gpt3-13b": ShardConfig("gpt3-13b", 5120, 40, 8, 0, 4, 2, 4, 2048, 20480, ARCH_GPT, index=2),
    "llama2-7b": ShardConfig("llama2-7b", 4096, 32, 8, 0, 2, 4, 2, 4096, 11008, ARCH_LLAMA, index=3),
    "llama2-13b": ShardConfig("llama2-13b", 5120, 40, 8, 0, 4, 4, 4, 4096, 13824, ARCH_LLAMA, index=4),
    # GPT-3 sizes of Table 1 that the list above lacks, at the same 2048-token context
    "gpt3-6.7b": ShardConfig("gpt3-6.7b", 4096, 32, 8, 0, 2, 2, 8, 2048, 16384, ARCH_GPT, index=20),
    "gpt3-30b": ShardConfig("gpt3-30b", 7168, 56, 8, 0, 4, 2, 4, 2048, 28672, ARCH_GPT, index=21),
    # the evaluation's own shapes (Sec. 5.3, 5.4): sequence length 512 or 1024, micro-batch 4 to 64
    "gpt3-13b-s512-mb4": ShardConfig("gpt3-13b-s512-mb4", 5120, 40, 8, 0, 2, 1, 4, 512, 20480, ARCH_GPT, index=22),
    "gpt3-13b-s1024-mb16": ShardConfig("gpt3-13b-s1024-mb16", 5120, 40, 8, 0, 4, 2, 16, 1024, 20480, ARCH_GPT, index=23),
    "gpt3-6.7b-s1024-mb32": ShardConfig("gpt3-6.7b-s1024-mb32", 4096, 32, 8, 0, 4, 2, 32, 1024, 16384, ARCH_GPT, index=24),
    "gpt3-2.7b-s512-mb64": ShardConfig("gpt3-2.7b-s512-mb64", 2560, 32, 8, 0, 4, 2, 64, 512, 10240, ARCH_GPT, index=25),
    "llama2-7b-s1024-mb16": ShardConfig("llama2-7b-s1024-mb16", 4096, 32, 8, 0, 4, 2, 16, 1024, 11008, ARCH_LLAMA, index=26),
    "llama2-13b-s512-mb16": ShardConfig("llama2-13b-s512-mb16", 5120, 40, 8, 0, 4, 2, 16, 512, 13824, ARCH_LLAMA, index=27),
    # a Llama-shaped toy that the oracle finishes at once (parity / pin cases only)
    "tiny-llama": ShardConfig("tiny-llama", 256, 4, 2, 0, 2, 2, 2, 128, 704, ARCH_LLAMA, index=5),
}


def round_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "value is not bf16-representable"
    return (u >> np.uint32(16)).astype(np.uint16)


def _rng(seed: int, tensor_id: int, rank: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, tensor_id, rank])))


def _normal(seed, tensor_id, rank, shape, std) -> np.ndarray:
    g = _rng(seed, tensor_id, rank)
    a = g.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return round_bf16(a)


# tensor ids (fixed: changing one changes every stored expectation)
_T_X, _T_DY = 1, 2
_T_WQKV, _T_BQKV, _T_WO, _T_WUP, _T_BUP, _T_WDOWN = 10, 11, 12, 13, 14, 15
_T_N1G, _T_N1B, _T_BO, _T_N2G, _T_N2B, _T_BDOWN = 20, 21, 22, 23, 24, 25
_T_AO, _T_MO, _T_D2O, _T_D1O = 30, 31, 32, 33

PARAM_NAMES = ("norm1_g", "norm1_b", "w_qkv", "b_qkv", "w_o", "b_o",
               "norm2_g", "norm2_b", "w_up", "b_up", "w_down", "b_down")


def config_seed(cfg: ShardConfig) -> int:
    return BASE_SEED + cfg.index


def make_activations(cfg: ShardConfig, seed: int | None = None):
    """x and dy, each [b, s, h] ~ N(0,1)."""
    seed = config_seed(cfg) if seed is None else seed
    shape = (cfg.batch, cfg.seq, cfg.hidden)
    return _normal(seed, _T_X, 0, shape, 1.0), _normal(seed, _T_DY, 0, shape, 1.0)


def make_others(cfg: ShardConfig, seed: int | None = None, scale: float = 0.5):
    """Stand-ins for what the four all-reduces would add from the other ranks."""
    seed = (config_seed(cfg) if seed is None else seed) + 1000
    shape = (cfg.batch, cfg.seq, cfg.hidden)
    return {
        "attn_others": _normal(seed, _T_AO, 0, shape, scale),
        "mlp_others": _normal(seed, _T_MO, 0, shape, scale),
        "dln2_others": _normal(seed, _T_D2O, 0, shape, scale),
        "dln1_others": _normal(seed, _T_D1O, 0, shape, scale),
    }


def make_rank_params(cfg: ShardConfig, rank: int | None = None, seed: int | None = None,
                     random_affine: bool = False, std: float = 0.02) -> Dict[str, np.ndarray | None]:
    """The twelve parameter tensors of rank ``rank`` (row-major [in, out] matrices).

    w_qkv [h, 3*h_l] with column blocks [Q | K | V], heads contiguous inside a block;
    w_o [h_l, h]; w_up [h, f_l] (GPT) or [h, 2*f_l] = [gate | up] (Llama); w_down [f_l, h].
    Replicated tensors (norm gains/shifts, b_o, b_down) do not depend on ``rank``.
    Llama has no shifts and no biases: those entries are None.
    """
    seed = config_seed(cfg) if seed is None else seed
    r = cfg.rank if rank is None else rank
    h, hl, fl = cfg.hidden, cfg.h_local, cfg.f_local
    llama = cfg.arch == ARCH_LLAMA
    P: Dict[str, np.ndarray | None] = {}
    P["w_qkv"] = _normal(seed, _T_WQKV, r, (h, 3 * hl), std)
    P["w_o"] = _normal(seed, _T_WO, r, (hl, h), std)
    P["w_up"] = _normal(seed, _T_WUP, r, (h, cfg.up_cols), std)
    P["w_down"] = _normal(seed, _T_WDOWN, r, (fl, h), std)
    ones = np.ones(h, dtype=np.float32)
    if random_affine:
        P["norm1_g"] = round_bf16(ones + _normal(seed, _T_N1G, 0, (h,), 0.1))
        P["norm2_g"] = round_bf16(ones + _normal(seed, _T_N2G, 0, (h,), 0.1))
    else:
        P["norm1_g"], P["norm2_g"] = ones.copy(), ones.copy()
    if llama:
        for k in ("norm1_b", "norm2_b", "b_qkv", "b_o", "b_up", "b_down"):
            P[k] = None
    elif random_affine:
        P["norm1_b"] = _normal(seed, _T_N1B, 0, (h,), 0.1)
        P["norm2_b"] = _normal(seed, _T_N2B, 0, (h,), 0.1)
        P["b_qkv"] = _normal(seed, _T_BQKV, r, (3 * hl,), std)
        P["b_up"] = _normal(seed, _T_BUP, r, (fl,), std)
        P["b_o"] = _normal(seed, _T_BO, 0, (h,), std)
        P["b_down"] = _normal(seed, _T_BDOWN, 0, (h,), std)
    else:
        P["norm1_b"] = np.zeros(h, np.float32)
        P["norm2_b"] = np.zeros(h, np.float32)
        P["b_qkv"] = np.zeros(3 * hl, np.float32)
        P["b_up"] = np.zeros(fl, np.float32)
        P["b_o"] = np.zeros(h, np.float32)
        P["b_down"] = np.zeros(h, np.float32)
    return P


LAYER_SEED_STRIDE = 7919


def make_stack(cfg: ShardConfig, nlayers: int, rank: int | None = None, random_affine: bool = False,
               std: float = 0.02, others_scale: float = 0.5):
    """Parameters and all-reduce stand-ins of ``nlayers`` blocks: block l draws from seed + l * 7919."""
    base = config_seed(cfg)
    params = [make_rank_params(cfg, rank, seed=base + l * LAYER_SEED_STRIDE, random_affine=random_affine, std=std)
              for l in range(nlayers)]
    others = [make_others(cfg, seed=base + l * LAYER_SEED_STRIDE, scale=others_scale) for l in range(nlayers)]
    return params, others
