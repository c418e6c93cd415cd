"""Timeline of one forward + backward step across the stream pool, from the library's own per-launch events
(domino_profile_record): which step of the path ran when on which stream, the gaps in front of a launch, and how
long the step had 0, 1, 2, ... launches in flight.  Device-memory plumbing only.

    python -m paper_2409_15241_amd.timeline --workload gpt3-13b --streams 4
"""
from __future__ import annotations

import argparse
import os

# one hardware queue per pool stream (see bench.py); only when this is the program: a process that imports the module
# may have started the HIP runtime already, which reads the variable once
if __name__ == "__main__" and int(os.environ.get("GPU_MAX_HW_QUEUES", "0") or 0) < 8:
    os.environ["GPU_MAX_HW_QUEUES"] = "8"


def record_step(buf, warm: int = 10):
    """Runs warm + 3 steps back to back, the last 3 with per-launch events, and returns the middle one as a list
    of (step class, stream handle, start ms, stop ms), times counted from the step's first start."""
    import torch
    from . import domino
    for _ in range(warm):
        buf.forward()
        buf.backward(accumulate=False)
    domino.domino_profile_reset()
    domino.domino_profile_enable(True)
    try:
        for _ in range(3):
            buf.forward()
            buf.backward(accumulate=False)
        torch.cuda.synchronize()
    finally:
        domino.domino_profile_enable(False)
    n = domino.domino_profile_records()
    recs = [domino.domino_profile_record(i) for i in range(n)]
    domino.domino_profile_reset()
    per = n // 3
    step = recs[per:2 * per]
    t0 = min(r[2] for r in step)
    return [(name, st, a - t0, b - t0) for name, st, a, b in step]


def in_flight(step):
    """{k: milliseconds of the step during which k launches were in flight}."""
    edges = sorted([(a, 1) for _, _, a, _ in step] + [(b, -1) for _, _, _, b in step])
    out, cur, last = {}, 0, edges[0][0]
    for t, d in edges:
        out[cur] = out.get(cur, 0.0) + (t - last)
        last, cur = t, cur + d
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="gpt3-13b")
    ap.add_argument("--streams", type=int, default=4)
    args = ap.parse_args()
    from . import domino, harness, synth, tune
    domino.load()
    sc = synth.WORKLOADS[args.workload]
    params, x, dy, others = tune.make_data(sc)
    buf = harness.LayerBuffers(sc, params, x, dy, others, streams=tune.stream_pool(args.streams))
    step = record_step(buf)
    print(f"{sc.name} p={sc.p} q={sc.q}: {len(step)} launches, span {max(r[3] for r in step) * 1e3:.0f} us "
          f"(with two event records per launch)")
    streams = {}
    for r in step:
        streams.setdefault(r[1], []).append(r)
    for k, rs in enumerate(streams.values()):
        rs.sort(key=lambda r: r[2])
        prev, cells = None, []
        for name, _, a, b in rs:
            gap = (a - prev) * 1e3 if prev is not None else a * 1e3
            cells.append(f"{name}@{a * 1e3:.0f}+{(b - a) * 1e3:.0f}" + (f"(gap {gap:.0f})" if gap > 8 else ""))
            prev = b
        print(f"stream {k}: " + "  ".join(cells))
    print("us with k launches in flight:", {k: round(v * 1e3) for k, v in sorted(in_flight(step).items())})


if __name__ == "__main__":
    main()
