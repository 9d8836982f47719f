#!/usr/bin/env python3
"""Benchmark of the DARK attention hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input:
a forward call of the configuration's entry point (dark_attn_fwd for the
bidirectional configurations, dark_attn_causal_fwd for the causal ones; the
finetuning configuration runs the training pair dark_attn_causal_fwd_save +
dark_attn_bwd_saved, in which the backward takes over the forward's key norms and
prefix states instead of recomputing them).  Inputs are resident in HBM before
the timed region; several distinct input copies are rotated so that the 256 MB
memory-side cache cannot serve a step's reads from the previous step.

Prints one JSON line (see the repository's design notes for the field meanings).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"hbm": (8000.0, "GB/s"), "mfma": (2500.0, "TFLOP/s"), "alu": (157.3, "TFLOP/s")}


def algorithmic_work(cfg):
    """Per-step algorithmic flops and HBM bytes of the forward pass (plus the backward pass where the
    configuration has one), and per kernel.

    Per token-head: projections of q and k through A = W M (2dm each), the norm terms
    (2dr each; the query-side one cancels in the ratio but is part of the definition),
    phi(K)^T [V|1] (2m(dv+1)) and phi(Q)[S|z] (2m(dv+1)).  Bytes: read Q, K, V, write out.
    Causal adds the within-chunk triangle: m(C+1) for the scores and (dv+1)(C+1) for their
    product with [V|1]."""
    th = cfg.B * cfg.H * cfg.L
    s_in = 2 if cfg.dtype == "bf16" else 4
    d, r, m, dv = cfg.d, cfg.r, cfg.m, cfg.dv
    f_tok = 4 * d * m + 4 * d * r + 4 * m * (dv + 1)
    if cfg.causal:
        f_tok += m * (cfg.chunk + 1) + (dv + 1) * (cfg.chunk + 1)
    b_tok = (2 * d + dv) * s_in + dv * s_in
    if cfg.backward:
        # Backward pass (a call of its own): every forward contraction has two gradient contractions of the same
        # size; it reads Q, K, V and dOut and writes dQ, dK, dV in fp32 (dM is a few KB per head).
        f_tok *= 3
        b_tok += (2 * d + dv) * s_in + dv * s_in + (2 * d + dv) * 4
    per_kernel = {
        # kernel name -> (bound, algorithmic units per launch) ; bytes for hbm, flops otherwise
        "fused_kv_reduce": ("hbm", th * (d + dv) * s_in),
        "fused_readout": ("hbm", th * (d + dv) * s_in),
        # the scan's MFMA work: both projections, the state read-out and update, the tile triangle
        "fused_causal_scan": ("mfma", th * (4 * d * m + 4 * m * (dv + 1) + m * (cfg.chunk + 1) + (dv + 1) * (cfg.chunk + 1))),
        "fused_causal_state": ("hbm", th * (d + dv) * s_in),
        "fused_key_norms": ("hbm", th * d * s_in),
        "f32_gemm": ("alu", th * f_tok),   # all GEMM launches of one step together
        # dark_featurize, per launch (one tensor): rows read once, features written once
        "fused_featurize": ("hbm", th * (d + m) * s_in),
        # dark_whiten: the second moments read every row of Q and K once (the per-head eigen-decomposition is
        # a fixed cost that does not grow with the number of rows)
        "whiten_moments": ("hbm", 2 * th * d * s_in),
        # dark_decode_step: the fp32 state of every (b,h) is read and written once
        "decode_step": ("hbm", 2 * cfg.B * cfg.H * m * (dv + 1) * 4),
        # backward, forward-order pass (tiles of T = 32 tokens): both projections, numerator and denominator
        # again, the logit gradients of the queries (state part and tile triangle), dQ, and the updates of
        # S, Rn and T_Q; reverse-order pass: projections, dV, the logit gradients of the keys, dK (with the
        # norm term through M'^T M'), and the updates of Rn, T_K and Rm
        "fused_bwd_fwd": ("mfma", th * (4 * d * m + 4 * m * (dv + 1) + 4 * m * d + 4 * m * dv + 33 * (2 * m + dv + 1))),
        "fused_bwd_rev": ("mfma", th * (4 * d * m + 6 * m * dv + 4 * m * d + 4 * d * r + 33 * (2 * m + dv))),
    }
    return th * f_tok, th * b_tok, per_kernel


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` on `workload`, from the committed rocprofv3 --pmc summary
    (FETCH_SIZE + WRITE_SIZE, each scaled by what the same counter reads for a plain copy of known
    size), or None when no such measurement is on file."""
    path = os.path.join(ROOT, traffic_file(workload))
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 2 and parts[0] == kernel and parts[1].startswith("hbm_bytes_per_launch="):
            return float(parts[1].split("=", 1)[1])
    return None


def traffic_file(workload):
    return os.path.join("profiles", f"hbm_traffic_{workload}.txt")


def measure_ceilings(dk, torch):
    """What this chip sustains right now with plain kernels: copy and read rates over 256 MiB buffers
    (rotated, so that the memory-side cache serves none of it) and a dense fp16 MFMA loop.  Timed with
    events on the stream the kernels run on, after the attention loops (clocks already settled)."""
    n = 64 * 1024 * 1024
    bufs = [torch.full((n,), float(k + 1), dtype=torch.float32, device="cuda") for k in range(3)]
    dsts = [torch.empty_like(bufs[0]) for _ in range(2)]
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")

    def timed(fn, reps, warm):
        for i in range(warm):
            fn(i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(reps):
            fn(i)
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    nb = n * 4
    t_copy = timed(lambda i: dk.ceiling_copy(dsts[i % 2], bufs[i % 3]), 24, 6)
    t_read = timed(lambda i: dk.ceiling_read(bufs[i % 3], sink), 24, 6)
    flops = dk.ceiling_mfma(1, sink)
    iters = 20000
    t_mfma = timed(lambda i: dk.ceiling_mfma(iters, sink), 6, 2)
    del bufs, dsts
    return {
        "copy_GBps": 2 * nb / t_copy / 1e9, "read_GBps": nb / t_read / 1e9,
        "mfma_f16_TFLOPs": flops * iters / t_mfma / 1e12,
        "how": "plain kernels of the library (dark_ceiling_*): 256 MiB copy (bytes read + written) and read, "
               "rotated buffers; 2048 waves x 4 independent chains of 32x32x16 fp16 MFMAs",
    }


def to_device(inp, bf16):
    """torch device tensors of a problem: bf16 tensors are built from the stored bit patterns."""
    import numpy as np
    import torch
    dev = {}
    for n in ("Q", "K", "V", "dOut"):
        if n not in inp:
            continue
        if bf16:
            dev[n] = torch.from_numpy(inp[n + "_bits"].view(np.int16)).view(torch.bfloat16).cuda()
        else:
            dev[n] = torch.from_numpy(inp[n]).cuda()
    dev["M"] = torch.from_numpy(inp["M"]).cuda()
    dev["W"] = torch.from_numpy(inp["W"]).cuda()
    return dev


def head(inp, b, h):
    W = inp["W"]
    return inp["Q"][b, h], inp["K"][b, h], inp["V"][b, h], inp["M"][h], (W if W.ndim == 2 else W[h])


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # Defaults long enough for the clocks to settle: the first milliseconds after an idle period run at a
    # transient clock (boost, then a dip while the power manager reacts), and a 25-step run lies entirely
    # inside that transient.  Steady state is reached after a few hundred steps of the headline workload.
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default: enough for about 0.3 s)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed warm-up steps (default: a quarter of --steps)")
    ap.add_argument("--config", type=int, default=2, help="benchmark configuration 1..5 (default 2, the headline)")
    ap.add_argument("--path", choices=["auto", "f32", "fused"], default="auto")
    ap.add_argument("--op", choices=["attn", "featurize", "whiten", "decode"], default="attn",
                    help="attn (default): the attention step the metric is quoted on; featurize: dark_featurize of "
                         "the configuration's Q (query contract) and K (key contract), a side measurement of that "
                         "entry point (value = rows/s); whiten: dark_whiten of the configuration's Q and K (value = rows/s); decode: "
                         "dark_decode_step, one token per (b,h) of the configuration per step (value = tokens/s)")
    ap.add_argument("--copies", type=int, default=3, help="distinct input copies rotated between steps")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every GPU box has one GPU); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2603_04127_amd as dk
    from paper_2603_04127_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    dk.lib()  # fail loudly if the HIP library is missing
    cfg = synth.CONFIGS[args.config]
    path = {"auto": dk.PATH_AUTO, "f32": dk.PATH_F32, "fused": dk.PATH_FUSED}[args.path]
    bf16 = cfg.dtype == "bf16"
    t0 = time.time()
    inp = synth.make_inputs(cfg)
    dev0 = to_device(inp, bf16)
    copies = []
    for k in range(max(1, args.copies)):
        c = dict(dev0)
        if k:
            for n in ("Q", "K", "V", "dOut"):
                if n in c:
                    # same distribution, different memory: rotate batch and sequence
                    c[n] = torch.roll(dev0[n], shifts=(k % max(cfg.B, 1), 17 * k), dims=(0, 2)).contiguous()
        c["out"] = torch.empty_like(c["V"])
        if args.op == "decode":
            # the recurrent state of every (b,h), filled by a short run of tokens; one more token per step
            c["state"] = dk.decode_state(cfg.B, cfg.H, cfg.m, cfg.dv)
            for t in range(4):
                dk.dark_decode_step(c["Q"][:, :, t].contiguous(), c["K"][:, :, t].contiguous(),
                                    c["V"][:, :, t].contiguous(), c["M"], c["W"], c["state"])
            c["q1"], c["k1"], c["v1"] = (c[n][:, :, 5].contiguous() for n in ("Q", "K", "V"))
            c["o1"] = torch.empty_like(c["v1"])
        if cfg.backward:
            f32 = dict(dtype=torch.float32, device="cuda")
            c["grads"] = {"dQ": torch.empty(c["Q"].shape, **f32), "dK": torch.empty(c["K"].shape, **f32),
                          "dV": torch.empty(c["V"].shape, **f32), "dM": torch.empty(c["M"].shape, **f32)}
        copies.append(c)
    gen_s = time.time() - t0

    def step(c):
        if args.op == "featurize":
            dk.dark_featurize(c["Q"], c["M"], c["W"], True, path=path)
            dk.dark_featurize(c["K"], c["M"], c["W"], False, path=path)
            return
        if args.op == "whiten":
            dk.dark_whiten(c["Q"], c["K"])
            return
        if args.op == "decode":
            dk.dark_decode_step(c["q1"], c["k1"], c["v1"], c["M"], c["W"], c["state"], out=c["o1"])
            return
        if cfg.causal and cfg.backward:
            # training step: the forward leaves its operand copies, key norms and prefix states to the backward
            _, saved = dk.dark_attn_causal_fwd_save(c["Q"], c["K"], c["V"], c["M"], c["W"], out=c["out"],
                                                    saved=c.get("saved"), chunk=cfg.chunk, path=path)
            c["saved"] = saved
            dk.dark_attn_bwd(c["Q"], c["K"], c["V"], c["M"], c["W"], c["dOut"], True, chunk=cfg.chunk, path=path,
                             saved=saved, grads=c["grads"])
            return
        if cfg.causal:
            dk.dark_attn_causal_fwd(c["Q"], c["K"], c["V"], c["M"], c["W"], out=c["out"], chunk=cfg.chunk, path=path)
        else:
            dk.dark_attn_fwd(c["Q"], c["K"], c["V"], c["M"], c["W"], out=c["out"], path=path)
        if cfg.backward:
            dk.dark_attn_bwd(c["Q"], c["K"], c["V"], c["M"], c["W"], c["dOut"], cfg.causal, chunk=cfg.chunk, path=path,
                             grads=c["grads"])

    if args.steps is None or args.warmup is None:
        # size the run from a short probe: about 0.3 s timed, a quarter of that as warm-up
        for i in range(3):
            step(copies[i % len(copies)])
        torch.cuda.synchronize()
        tp = time.perf_counter()
        for i in range(10):
            step(copies[i % len(copies)])
        torch.cuda.synchronize()
        per = (time.perf_counter() - tp) / 10
        if args.steps is None:
            args.steps = int(min(5000, max(20, 0.3 / per)))
        if args.warmup is None:
            args.warmup = max(5, args.steps // 4)
    for i in range(args.warmup):
        step(copies[i % len(copies)])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(args.steps):
        step(copies[i % len(copies)])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t1
    ms = dt / args.steps * 1e3
    tokens = cfg.B * cfg.L
    flops, nbytes, per_kernel = algorithmic_work(cfg)
    if args.op == "featurize":
        # two tensors of B*H*L rows each: projections (2dm + 2dr flops per row), rows in, features out
        th = cfg.B * cfg.H * cfg.L
        flops = 2 * th * (2 * cfg.d * cfg.m + 2 * cfg.d * cfg.r)
        nbytes = 2 * per_kernel["fused_featurize"][1]
    if args.op == "whiten":
        th = cfg.B * cfg.H * cfg.L
        flops = 2 * th * 2 * cfg.d * cfg.d
        nbytes = per_kernel["whiten_moments"][1]
    if args.op == "decode":
        flops = cfg.B * cfg.H * (4 * cfg.d * cfg.r + 4 * cfg.r * cfg.m + 4 * cfg.m * (cfg.dv + 1))
        nbytes = per_kernel["decode_step"][1]

    # Per-kernel device time: a second loop in which the library attaches start/stop events to every
    # launch (stamped with the kernel's own begin and end on the launch stream; the stream is drained
    # before each timed launch, so this loop is slower than the timed region above).
    dk.timing_reset()
    dk.timing_enable(True)
    ksteps = min(args.steps, 200)
    for i in range(ksteps):
        step(copies[i % len(copies)])
    torch.cuda.synchronize()
    kt = dk.timing_read()
    dk.timing_enable(False)
    kernels = {k: {"launches": n, "avg_us": 1e3 * t / n, "us_per_step": 1e3 * t / ksteps} for k, (n, t) in kt.items()}
    dom = max(kt.items(), key=lambda kv: kv[1][1])[0]
    if args.op == "whiten":
        dom = "whiten_moments"   # the part that scales with the data; the eigen-decomposition is a fixed cost per head
    bound, units = per_kernel.get(dom, ("hbm", nbytes))
    us_step = kernels[dom]["us_per_step"]
    peak, unit = PEAK[bound]
    achieved = units / (us_step * 1e-6) / (1e9 if bound == "hbm" else 1e12)
    traffic = measured_traffic(cfg.name, dom)
    roofline = {"bound": bound, "kernel": dom, "achieved": achieved, "peak": peak, "unit": unit,
                "frac": achieved / peak, "traffic": traffic,
                "traffic_source": traffic_file(cfg.name) if traffic is not None else None,
                "avg_kernel_us": kernels[dom]["avg_us"], "launches_per_step": kernels[dom]["launches"] / ksteps}
    for k in kernels:
        tb = measured_traffic(cfg.name, k)
        if tb is not None:
            kernels[k]["hbm_bytes_per_launch"] = tb
    ceilings = measure_ceilings(dk, torch)
    measured_peak = {"hbm": ceilings["read_GBps"], "mfma": ceilings["mfma_f16_TFLOPs"]}.get(bound)
    if measured_peak:
        roofline["frac_of_measured_ceiling"] = achieved / measured_peak

    line = {
        "metric": ("DARK attention fwd tokens/sec and TFLOP/s; % of MFMA/HBM roofline (1 GPU)" if args.op == "attn"
                   else "dark_featurize rows/sec (query rows + key rows); % of MFMA/HBM roofline (1 GPU)" if args.op == "featurize"
                   else "dark_whiten rows/sec (query rows + key rows); % of HBM roofline (1 GPU)" if args.op == "whiten"
                   else "dark_decode_step tokens/sec (one token per batch entry, all heads); % of HBM roofline (1 GPU)"),
        "value": (tokens if args.op == "attn" else cfg.B if args.op == "decode" else 2 * cfg.B * cfg.H * cfg.L) / (ms * 1e-3),
        "unit": "tokens/s" if args.op in ("attn", "decode") else "rows/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "B": cfg.B, "H": cfg.H, "L": cfg.L, "d": cfg.d, "m": cfg.m, "dv": cfg.dv,
                   "causal": cfg.causal, "backward": cfg.backward, "path": args.path, "input_copies": len(copies),
                   "op": args.op},
        "tflops": flops / (ms * 1e-3) / 1e12,
        "algorithmic_gbps": nbytes / (ms * 1e-3) / 1e9,
        "step_frac_of_binding_roofline": max(flops / 2.5e15, nbytes / 8e12) / (ms * 1e-3),
        "step_frac_of_measured_ceilings": None,
        "roofline": roofline,
        "ceilings": ceilings,
        "kernels": kernels,
        "input_generation_s": gen_s,
    }

    line["step_frac_of_measured_ceilings"] = max(flops / (ceilings["mfma_f16_TFLOPs"] * 1e12),
                                                 nbytes / (ceilings["copy_GBps"] * 1e9)) / (ms * 1e-3)
    if not args.no_cpu_baseline and args.op == "attn":
        # The oracle as it stands, on a bounded sample of the same workload: whole heads of batch 0
        # until about --cpu-seconds of CPU time have been spent.
        from oracle import dark_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        heads = 0
        t2 = time.perf_counter()
        while (time.perf_counter() - t2) < args.cpu_seconds:
            b, h = divmod(heads % (cfg.B * cfg.H), cfg.H)
            Q, K, V, M, W = head(inp, b, h)
            Ls = min(cfg.L, 8192)     # causal oracle is a per-token loop: bound the sample length
            if cfg.causal:
                O.attn_causal(Q[:Ls], K[:Ls], V[:Ls], M, W)
            else:
                Ls = cfg.L
                O.attn_bidir(Q, K, V, M, W)
            heads += 1
        el = time.perf_counter() - t2
        line["cpu_baseline"] = {
            "value": (heads * Ls / cfg.H) / el, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"{heads} (b,h) slices (cycling over the {cfg.B * cfg.H} of the workload) of {Ls} positions of "
                      f"{cfg.name}, fp64 numpy oracle, forward only, {el:.1f} s; scaled by 1/H to tokens",
        }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
