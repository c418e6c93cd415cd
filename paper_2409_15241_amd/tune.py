"""Grid search of the partition granularity (Sec. 3.1, 5.3: before training, the system is benchmarked over
the row split p and the column split q and the fastest setting is kept).  On one GPU the measured
quantity is the time of the rank-local forward + backward of one block; the stream-pool size is a
third axis.  Device-memory plumbing only: every measured step runs through the C ABI.

    python -m paper_2409_15241_amd.tune --workload gpt3-13b
"""
from __future__ import annotations

import argparse
import json
import os
import time
from typing import Iterable, List, Optional, Tuple

if int(os.environ.get("GPU_MAX_HW_QUEUES", "0") or 0) < 8:   # one hardware queue per pool stream (see bench.py)
    os.environ["GPU_MAX_HW_QUEUES"] = "8"


def candidates(sc, ps: Iterable[int] = (1, 2, 4, 8), qs: Iterable[int] = (1, 2, 4)) -> List[Tuple[int, int]]:
    """The (p, q) pairs that cut this shard exactly: batch % p == 0 and hidden % q == 0 with hidden/q a
    multiple of 8 (the library's requirement)."""
    out = []
    for p in ps:
        for q in qs:
            if sc.batch % p == 0 and sc.hidden % q == 0 and (sc.hidden // q) % 8 == 0:
                out.append((p, q))
    return out


def measure(sc, nstreams: int, steps: int = 10, warmup: int = 3) -> float:
    """Milliseconds per forward + backward of the shard `sc` (its p and q) on a pool of nstreams streams."""
    import torch
    from . import harness, synth
    params = synth.make_rank_params(sc)
    x, dy = synth.make_activations(sc)
    buf = harness.LayerBuffers(sc, params, x, dy, synth.make_others(sc), nstreams=nstreams)
    for _ in range(warmup):
        buf.forward()
        buf.backward(accumulate=False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        buf.forward()
        buf.backward(accumulate=False)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def tune(sc, pairs: Optional[List[Tuple[int, int]]] = None, streams: Iterable[int] = (1, 2, 4),
         steps: int = 10, warmup: int = 3):
    """Returns (best, table): best = (p, q, nstreams, ms); table lists every measured setting."""
    table = []
    for (p, q) in (pairs if pairs is not None else candidates(sc)):
        for ns in streams:
            if ns > max(p, 1) and ns > 1:
                continue          # more streams than row slices adds nothing (column pieces stay on their slice's stream)
            ms = measure(sc.replace(p=p, q=q), ns, steps, warmup)
            table.append((p, q, ns, ms))
    best = min(table, key=lambda r: r[3])
    return best, table


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="gpt3-13b")
    ap.add_argument("--steps", type=int, default=10)
    args = ap.parse_args()
    from . import domino, synth
    domino.load()
    sc = synth.WORKLOADS[args.workload]
    best, table = tune(sc, steps=args.steps)
    for (p, q, ns, ms) in table:
        print(f"p={p} q={q} streams={ns}: {ms:8.3f} ms")
    print(json.dumps({"workload": sc.name, "best": {"p": best[0], "q": best[1], "streams": best[2], "ms": best[3]}}))


if __name__ == "__main__":
    main()
