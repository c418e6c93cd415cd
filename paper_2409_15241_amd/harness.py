"""Device-memory plumbing around the C ABI: uploads synthetic inputs, allocates the caller-owned
buffers with torch, owns the fixed stream pool, and calls domino_layer_fwd / domino_layer_bwd.
No arithmetic of the method happens here."""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

from . import domino, synth


def to_device_bf16(a: Optional[np.ndarray], device="cuda:0") -> Optional[torch.Tensor]:
    """float32 array of bf16-representable values -> bf16 device tensor (bit-exact)."""
    if a is None:
        return None
    bits = synth.bf16_bits(a).view(np.int16)
    return torch.from_numpy(bits).to(device).view(torch.bfloat16)


def to_host_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float32).numpy().astype(np.float64)


class LayerBuffers:
    """Everything one rank needs for forward + backward of one block, resident on the GPU."""

    def __init__(self, sc: synth.ShardConfig, params: Dict[str, Optional[np.ndarray]], x: np.ndarray,
                 dy: np.ndarray, others: Optional[Dict[str, np.ndarray]] = None, nstreams: int = 4,
                 device: str = "cuda:0", want_y: bool = True, streams=None):
        self.sc = sc
        self.cfg = domino.make_cfg(sc)
        rc = domino.domino_validate_cfg(self.cfg)
        if rc != domino.OK:
            raise domino.DominoError(rc, domino.domino_last_error())
        self.device = torch.device(device)
        dev = self.device
        self.params = {k: to_device_bf16(v, dev) for k, v in params.items()}
        self.x = to_device_bf16(x, dev)
        self.dy = to_device_bf16(dy, dev)
        oth = others or {}
        self.attn_others = to_device_bf16(oth.get("attn_others"), dev)
        self.mlp_others = to_device_bf16(oth.get("mlp_others"), dev)
        self.dln2_others = to_device_bf16(oth.get("dln2_others"), dev)
        self.dln1_others = to_device_bf16(oth.get("dln1_others"), dev)
        shape = (sc.batch, sc.seq, sc.hidden)
        mk = lambda: torch.empty(shape, dtype=torch.bfloat16, device=dev)
        self.attn_partial, self.mlp_partial = mk(), mk()
        self.y = mk() if want_y else None
        self.dln2_partial, self.dln1_partial, self.dx = mk(), mk(), mk()
        self.saved = torch.empty(domino.domino_saved_bytes(self.cfg), dtype=torch.uint8, device=dev)
        self.workspace = torch.empty(domino.domino_workspace_bytes(self.cfg), dtype=torch.uint8, device=dev)
        self.grads = {k: (None if v is None else torch.zeros(v.shape, dtype=torch.float32, device=dev))
                      for k, v in self.params.items()}
        # fixed pool of streams created once and picked by index (default priority); a caller that builds many
        # of these objects passes its own pool so that the streams (and their hardware queues) stay the same
        self.streams = list(streams) if streams is not None else [torch.cuda.Stream(device=dev) for _ in range(nstreams)]
        # the uploads and fills above were enqueued on torch's current stream, which the pool's streams
        # do not wait for: everything must have landed before the first library call reads it
        torch.cuda.synchronize(dev)

    def forward(self) -> None:
        domino.domino_layer_fwd(self.cfg, self.params, self.x, self.attn_others, self.mlp_others,
                                self.attn_partial, self.mlp_partial, self.y, self.saved, self.workspace,
                                self.streams)

    def backward(self, accumulate: bool = False) -> None:
        domino.domino_layer_bwd(self.cfg, self.params, self.saved, self.x, self.dy, self.dln2_others,
                                self.dln1_others, self.dln2_partial, self.dln1_partial, self.dx,
                                self.grads, accumulate, self.workspace, self.streams)

    def sync(self) -> None:
        torch.cuda.synchronize(self.device)

    def saved_tensor(self, name: str) -> torch.Tensor:
        """A named tensor inside the saved block as a flat device tensor (bf16, or fp32 for statistics)."""
        off, size = domino.domino_saved_slot(self.cfg, name)
        raw = self.saved[off:off + size]
        if name in ("lse", "mean1", "rstd1", "mean2", "rstd2"):
            return raw.view(torch.float32)
        return raw.view(torch.bfloat16)


class StackBuffers:
    """A stack of blocks of one configuration, resident on the GPU: per block its parameters, the four
    stand-ins of the other ranks' sums, the four partial outputs, y, the saved activations and the gradients."""

    def __init__(self, sc: synth.ShardConfig, params, x: np.ndarray, dy: np.ndarray, others=None,
                 nstreams: int = 4, device: str = "cuda:0", streams=None):
        self.sc = sc
        self.cfg = domino.make_cfg(sc)
        rc = domino.domino_validate_cfg(self.cfg)
        if rc != domino.OK:
            raise domino.DominoError(rc, domino.domino_last_error())
        self.device = torch.device(device)
        dev = self.device
        self.nlayers = len(params)
        self.params = [{k: to_device_bf16(v, dev) for k, v in P.items()} for P in params]
        self.x = to_device_bf16(x, dev)
        self.dy = to_device_bf16(dy, dev)
        others = others or [{} for _ in params]
        self.others = [{k: to_device_bf16(v, dev) for k, v in o.items()} for o in others]
        shape = (sc.batch, sc.seq, sc.hidden)
        mk = lambda: torch.empty(shape, dtype=torch.bfloat16, device=dev)
        nbytes = domino.domino_saved_bytes(self.cfg)
        self.out = [dict(attn_partial=mk(), mlp_partial=mk(), y=mk(), dln2_partial=mk(), dln1_partial=mk(),
                         saved=torch.empty(nbytes, dtype=torch.uint8, device=dev)) for _ in params]
        self.dx = mk()
        self.workspace = torch.empty(domino.domino_stack_workspace_bytes(self.cfg, self.nlayers), dtype=torch.uint8,
                                     device=dev)
        self.grads = [{k: (None if v is None else torch.zeros(v.shape, dtype=torch.float32, device=dev))
                       for k, v in P.items()} for P in self.params]
        self.streams = list(streams) if streams is not None else [torch.cuda.Stream(device=dev) for _ in range(nstreams)]
        torch.cuda.synchronize(dev)     # uploads ran on torch's current stream, which the pool does not wait for

    def layer_input(self, l: int) -> torch.Tensor:
        return self.x if l == 0 else self.out[l - 1]["y"]

    def forward(self) -> None:
        io = [dict(attn_others=o.get("attn_others"), mlp_others=o.get("mlp_others"), attn_partial=b["attn_partial"],
                   mlp_partial=b["mlp_partial"], y=b["y"], saved=b["saved"]) for o, b in zip(self.others, self.out)]
        domino.domino_stack_fwd(self.cfg, self.params, self.x, io, self.workspace, self.streams)

    def backward(self, accumulate: bool = False) -> None:
        io = [dict(x=self.layer_input(l), saved=b["saved"], dln2_others=o.get("dln2_others"),
                   dln1_others=o.get("dln1_others"), dln2_partial=b["dln2_partial"], dln1_partial=b["dln1_partial"])
              for l, (o, b) in enumerate(zip(self.others, self.out))]
        domino.domino_stack_bwd(self.cfg, self.params, self.dy, io, self.dx, self.grads, accumulate, self.workspace,
                                self.streams)

    def sync(self) -> None:
        torch.cuda.synchronize(self.device)
