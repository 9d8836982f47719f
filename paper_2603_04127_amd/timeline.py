"""Wall-clock timeline of the two large kernels of the bidirectional MFMA forward (key/value pass, readout)
at benchmark configuration 2.

    python -m paper_2603_04127_amd.timeline [--no-build]

Builds libdark_timeline.so beside the ordinary library (same sources, -DDARK_TIMELINE: every wave stores the
device's 100 MHz wall clock at fixed points of its run), runs the forward on the synthetic inputs of the
configuration and prints, in microseconds since the first wave of the kernel started, when the waves reached
each point.  Measurement only: the instrumented kernels run within about 1 % of the ordinary ones."""
from __future__ import annotations

import argparse
import os
import sys

import numpy as np


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--no-build", action="store_true", help="use an existing libdark_timeline.so")
    args = ap.parse_args()
    from paper_2603_04127_amd import build as B
    if not args.no_build or not os.path.exists(B.LIB_TIMELINE):
        B.build(verbose=False, timeline=True)
    import paper_2603_04127_amd as dk
    dk.LIB_PATH = B.LIB_TIMELINE
    import torch
    from paper_2603_04127_amd import synth

    cfg = synth.CONFIGS[2]
    inp = synth.make_inputs(cfg)
    dev = {n: torch.from_numpy(inp[n + "_bits"].view(np.int16)).view(torch.bfloat16).cuda() for n in ("Q", "K", "V")}
    dev["M"], dev["W"] = torch.from_numpy(inp["M"]).cuda(), torch.from_numpy(inp["W"]).cuda()
    out = torch.empty_like(dev["V"])

    def step():
        dk.dark_attn_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], out=out)

    for _ in range(200):  # settle the clocks
        step()
    torch.cuda.synchronize()
    dk.timing_reset()
    dk.timing_enable(True)
    for _ in range(20):
        step()
    torch.cuda.synchronize()
    kt = dk.timing_read()
    dk.timing_enable(False)
    print("kernel durations of the instrumented build (events, us):",
          {k: round(1e3 * t / n, 1) for k, (n, t) in kt.items()})
    step()
    torch.cuda.synchronize()

    def us(a):
        a = a.astype(np.float64)
        return (a - a[..., 0].min()) * 0.01  # 100 MHz ticks

    def line(name, v):
        print(f"  {name:28s} mean {v.mean():6.2f}  min {v.min():6.2f}  median {np.median(v):6.2f}  max {v.max():6.2f}")

    kv = us(np.array(dk.timeline_read(0, 480 * 4 * 16), dtype=np.int64).reshape(480, 4, 16))
    print("key/value pass, 480 workgroups x 4 waves (two workgroups per CU; the first 256 are the first residents):")
    for nm, i in (("kernel start", 0), ("M' in LDS", 1), ("first barrier passed", 2), ("tile loop begins", 3),
                  ("tile loop done", 4), ("kernel end", 5)):
        line(nm, kv[:, :, i])
    for nm, sl in (("first residents (0..223)", slice(0, 224)), ("alone on their CU (224..255)", slice(224, 256)),
                   ("second residents (256..479)", slice(256, 480))):
        v = kv[sl]
        print(f"  {nm:28s} loop begins {v[:, :, 3].mean():5.2f}, loop {np.mean(v[:, :, 4] - v[:, :, 3]):5.2f} us, ends {v[:, :, 5].mean():5.2f}")
    ro = us(np.array(dk.timeline_read(1, 256 * 8 * 16), dtype=np.int64).reshape(256, 8, 16))
    print("readout, 256 workgroups x 8 waves (waves 0-3 are the older wave of their SIMD), three items per wave:")
    names = ["kernel start", "first fill done"]
    for i in range(3):
        names += [f"item {i}: unit loop begins", f"item {i}: unit loop done", f"item {i}: rows stored"]
    for k, nm in enumerate(names):
        line(nm, ro[:, :, k])
    line("kernel end", ro[:, :, 15])
    for nm, sl in (("older waves (0-3)", slice(0, 4)), ("younger waves (4-7)", slice(4, 8))):
        v = ro[:, sl]
        loops = np.mean([v[:, :, 3 + 3 * i] - v[:, :, 2 + 3 * i] for i in range(3)])
        print(f"  {nm:28s} unit loop {loops:5.2f} us per item, end {v[:, :, 15].mean():5.2f}")
    return 0


if __name__ == "__main__":
    sys.exit(main())
