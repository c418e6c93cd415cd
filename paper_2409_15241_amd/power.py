"""Board power while the path runs: `python -m paper_2409_15241_amd.power [--workload gpt3-13b] [--seconds 3]`.

Samples the GPU's power sensor (hwmon `power1_input`, the same figure `rocm-smi --showpower` prints) while, one
after the other, each of these runs back to back for a few seconds: nothing (idle), the MFMA-only probe, the
library's GEMM at 8192^3 in its three operand layouts, a plain device copy of known size, and forward + backward of
the workload's block as bench.py times it.  Prints time per launch, mean power, energy per launch and what that is
per flop or per byte above the idle power.  Under sustained matrix load an MI355X sits at its power cap, so that
the time of a step is its energy over the cap: this table says where the energy goes."""
from __future__ import annotations

import argparse
import glob
import os
import threading
import time

# one hardware queue per pool stream (see bench.py); only when this is the program: a process that imports the module
# may have started the HIP runtime already, which reads the variable once
if __name__ == "__main__" and int(os.environ.get("GPU_MAX_HW_QUEUES", "0") or 0) < 8:
    os.environ["GPU_MAX_HW_QUEUES"] = "8"


def sensor():
    for pat in ("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input",
                "/sys/class/drm/card*/device/hwmon/hwmon*/power1_average"):
        found = sorted(glob.glob(pat))
        if found:
            return found[0]
    raise RuntimeError("no hwmon power sensor found for the GPU")


def read_watts(path):
    with open(path) as fh:
        return int(fh.read()) / 1e6


class Sampler:
    """Mean of the sensor readings between start() and stop(), skipping the first `settle` seconds."""

    def __init__(self, path, settle=1.0, period=0.05):
        self.path, self.settle, self.period = path, settle, period
        self.samples, self._stop, self._th = [], False, None

    def _run(self):
        t0 = time.perf_counter()
        while not self._stop:
            w = read_watts(self.path)
            if time.perf_counter() - t0 >= self.settle:
                self.samples.append(w)
            time.sleep(self.period)

    def start(self):
        self.samples, self._stop = [], False
        self._th = threading.Thread(target=self._run)
        self._th.start()

    def stop(self):
        self._stop = True
        self._th.join()
        return sum(self.samples) / max(1, len(self.samples)), max(self.samples or [0.0])


def soak(torch, fn, seconds, batch=20):
    """fn() enqueued back to back for `seconds`; returns seconds per call."""
    fn()
    torch.cuda.synchronize()
    n, t0 = 0, time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(batch):
            fn()
        torch.cuda.synchronize()
        n += batch
    return (time.perf_counter() - t0) / n


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="gpt3-13b")
    ap.add_argument("--seconds", type=float, default=3.0)
    ap.add_argument("--streams", type=int, default=4)
    args = ap.parse_args()
    import torch
    from paper_2409_15241_amd import domino, harness, synth
    import bench
    domino.load()
    path = sensor()
    cap = path.rsplit("/", 1)[0] + "/power1_cap"
    print(f"sensor {path}; power cap {read_watts(cap):.0f} W" if os.path.exists(cap) else f"sensor {path}")
    smp = Sampler(path)
    torch.cuda.init()
    torch.zeros(1, device="cuda")
    smp.start()
    time.sleep(args.seconds)
    idle, _ = smp.stop()
    rows = [("idle (context created, nothing running)", 0.0, idle, None, None)]

    def run(name, fn, flops=None, nbytes=None, batch=20):
        smp.start()
        dt = soak(torch, fn, args.seconds, batch)
        mean, peak = smp.stop()
        rows.append((name, dt, mean, flops, nbytes))
        unit = ""
        if flops:
            unit = f"{flops / dt / 1e12:8.1f} TFLOP/s  {(mean - idle) * dt / flops * 1e12:6.3f} pJ/flop above idle"
        if nbytes:
            unit = f"{nbytes / dt / 1e12:8.2f} TB/s     {(mean - idle) * dt / nbytes * 1e12:6.1f} pJ/B above idle"
        print(f"{name:58s} {dt * 1e6:9.1f} us  {mean:6.0f} W (max {peak:4.0f})  {mean * dt:8.4f} J  {unit}", flush=True)

    print(f"{'idle':58s} {'':9s}     {idle:6.0f} W")
    g = torch.Generator(device="cuda").manual_seed(20240915)
    a = torch.randn(2048, device="cuda", generator=g).to(torch.bfloat16)
    b = (0.02 * torch.randn(2048, device="cuda", generator=g)).to(torch.bfloat16)
    z = torch.zeros(2048, device="cuda", dtype=torch.bfloat16)
    out = torch.empty(512 * 256, device="cuda", dtype=torch.float32)
    st = torch.cuda.current_stream()
    iters = 4000
    fl = 512 * 4.0 * iters * 8 * 2 * 32 * 32 * 16
    run("MFMA only, N(0,1) x N(0,0.02) fragments", lambda: domino.domino_mfma_probe(a, b, out, 512, iters, st), flops=fl, batch=5)
    run("MFMA only, all-zero fragments", lambda: domino.domino_mfma_probe(z, z, out, 512, iters, st), flops=fl, batch=5)
    n = 8192
    A = torch.randn(n, n, device="cuda", generator=g).to(torch.bfloat16)
    B = (0.02 * torch.randn(n, n, device="cuda", generator=g)).to(torch.bfloat16)
    Cb = torch.empty(n, n, device="cuda", dtype=torch.bfloat16)
    Cf = torch.zeros(n, n, device="cuda", dtype=torch.float32)
    for name, lay, epi, Cm, beta in (("GEMM 8192^3 NN (forward product), 256x256 tile", domino.GEMM_NN, domino.EPI_STORE, Cb, 0),
                                     ("GEMM 8192^3 NT (input gradient), 256x256 tile", domino.GEMM_NT, domino.EPI_STORE, Cb, 0),
                                     ("GEMM 8192^3 TN (weight gradient, fp32 +=), 256x256 tile", domino.GEMM_TN, domino.EPI_ACC_F32, Cf, 1)):
        run(name, lambda lay=lay, epi=epi, Cm=Cm, beta=beta: domino.domino_gemm(lay, epi, 2, A, n, B, n, Cm, n, n, n, n, beta=beta, stream=st),
            flops=2.0 * n ** 3, batch=10)
    del A, B, Cb, Cf
    for mib in (1024, 64):
        src = torch.empty(mib << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        run(f"device copy of {mib} MiB (reads and writes that much)", lambda: dst.copy_(src), nbytes=2.0 * (mib << 20))
        del src, dst
    sc = synth.WORKLOADS[args.workload]
    params, x, dy, others = bench.draw_inputs(sc)
    buf = harness.LayerBuffers(sc, params, x, dy, others, nstreams=args.streams)

    def step():
        buf.forward()
        buf.backward(accumulate=False)
    run(f"{sc.name} block forward + backward (p={sc.p}, q={sc.q}, {args.streams} streams)", step,
        flops=bench.algorithmic_flops(sc), batch=10)


if __name__ == "__main__":
    main()
