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

# one hardware queue per pool stream (see bench.py); only when this is the program: a process that imports the module
# may have started the HIP runtime already, which reads the variable once
if __name__ == "__main__" and int(os.environ.get("GPU_MAX_HW_QUEUES", "0") or 0) < 8:
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


def make_data(sc):
    """The synthetic inputs of a shard; they do not depend on p, q or the pool, so a search draws them once."""
    from . import synth
    x, dy = synth.make_activations(sc)
    return synth.make_rank_params(sc), x, dy, synth.make_others(sc)


_POOL = []


def stream_pool(n: int):
    """The first n streams of one pool that lives as long as the process (Sec. 4.3.1: created once, picked by
    index), so that every measured setting runs on the same streams and hardware queues."""
    import torch
    while len(_POOL) < n:
        _POOL.append(torch.cuda.Stream())
    return _POOL[:n]


def measure(sc, nstreams: int, steps: int = 10, warmup: int = 3, data=None) -> float:
    """Milliseconds per forward + backward of the shard `sc` (its p and q) on a pool of nstreams streams."""
    import torch
    from . import harness
    params, x, dy, others = data if data is not None else make_data(sc)
    buf = harness.LayerBuffers(sc, params, x, dy, others, streams=stream_pool(nstreams))
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


def tune(sc, pairs: Optional[List[Tuple[int, int]]] = None, streams: Iterable[int] = (1, 2, 4, 8),
         steps: int = 10, warmup: int = 3, report=None):
    """Returns (best, table): best = (p, q, nstreams, ms); table lists every measured setting; report(row) is
    called after each measurement."""
    table = []
    data = make_data(sc)
    for (p, q) in (pairs if pairs is not None else candidates(sc)):
        for ns in streams:
            if ns > 1 and ns > (2 * p if p <= 2 else p):
                continue          # streams the library would not use: one per row slice, and with one or two slices
                                  # a second one per slice for the backward's weight gradients
            ms = measure(sc.replace(p=p, q=q), ns, steps, warmup, data)
            table.append((p, q, ns, ms))
            if report:
                report(table[-1])
    best = min(table, key=lambda r: r[3])
    return best, table


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="gpt3-13b", help="a name of synth.WORKLOADS, or 'all'")
    ap.add_argument("--steps", type=int, default=10)
    args = ap.parse_args()
    from . import domino, synth
    domino.load()
    names = [n for n in synth.WORKLOADS if not n.startswith("tiny")] if args.workload == "all" else [args.workload]
    for name in names:
        sc = synth.WORKLOADS[name]
        best, table = tune(sc, steps=args.steps, report=lambda r: print(
            f"{name}: p={r[0]} q={r[1]} streams={r[2]}: {r[3]:8.3f} ms", flush=True))
        print(json.dumps({"workload": sc.name, "best": {"p": best[0], "q": best[1], "streams": best[2], "ms": best[3]},
                          "as_configured": {"p": sc.p, "q": sc.q}}), flush=True)


if __name__ == "__main__":
    main()
