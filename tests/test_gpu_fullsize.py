"""Parity at the full benchmark sizes, in the launch configuration bench.py times, on sampled
(b, h) slices the oracle can compute in seconds."""
import numpy as np
import pytest

import paper_2603_04127_amd as dk
from paper_2603_04127_amd import synth
from oracle import dark_oracle as O
from tests import parity_util as U

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _np(t):
    return t.detach().float().cpu().numpy()


@pytest.mark.parametrize("n,heads", [(2, [(0, 0), (3, 7), (7, 11)]), (4, [(0, 5)])])
def test_bidirectional_configs(n, heads):
    cfg = synth.CONFIGS[n]
    inp = synth.make_inputs(cfg)
    dev = U.to_device(inp, True)
    out = dk.dark_attn_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"])
    torch.cuda.synchronize()
    for b, h in heads:
        want = O.attn_bidir(*U.head(inp, b, h))
        e = U.assert_close(_np(out[b, h]), want, U.TOL["bf16"], f"config {n} head {(b, h)}")
        print(f"config {n} head {(b, h)}: {U.fmt(e)}")


def test_causal_config3():
    cfg = synth.CONFIGS[3]
    inp = synth.make_inputs(cfg)
    dev = U.to_device(inp, True)
    out = dk.dark_attn_causal_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], chunk=cfg.chunk)
    torch.cuda.synchronize()
    rows = sorted(set([0, 1, 127, 128, 129, 4095, 4096, 8191] + list(range(5, cfg.L, 97))))
    for b, h in [(0, 0), (3, 15)]:
        want = O.attn_causal(*U.head(inp, b, h), rows=rows)
        e = U.assert_close(_np(out[b, h])[rows], want, U.TOL["bf16"], f"config 3 head {(b, h)}")
        print(f"config 3 head {(b, h)}: {U.fmt(e)}")


@pytest.mark.parametrize("path", ["fused", "f32"])
def test_finetune_config5(path):
    """Forward + backward at the finetuning configuration; the backward through the MFMA kernels (what
    DARK_PATH_AUTO and bench.py run) and through the fp32 kernels."""
    cfg = synth.CONFIGS[5]
    inp = synth.make_inputs(cfg)
    dev = U.to_device(inp, True)
    out = dk.dark_attn_causal_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], chunk=cfg.chunk)
    g = dk.dark_attn_bwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], dev["dOut"], True, chunk=cfg.chunk,
                         path=dk.PATH_FUSED if path == "fused" else dk.PATH_F32)
    torch.cuda.synchronize()
    for t in g.values():
        assert bool(torch.isfinite(t).all())
    check = U.assert_close_grad if path == "fused" else U.assert_close
    show = U.fmt_grad if path == "fused" else U.fmt
    h = 4
    dM = np.zeros((cfg.r, cfg.d))
    for b in range(cfg.B):
        Q, K, V, M, W = U.head(inp, b, h)
        dQ, dK, dV, dMb = O.attn_bwd_brute(Q, K, V, M, W, inp["dOut"][b, h], True)
        dM += dMb
        if b == 0:
            U.assert_close(_np(out[b, h]), O.attn_brute(Q, K, V, M, W, True), U.TOL["bf16"], "config 5 out")
        for name, want in (("dQ", dQ), ("dK", dK), ("dV", dV)):
            e = check(_np(g[name][b, h]), want, U.TOL["bf16"], f"config 5 {name}[{b},{h}] ({path})")
            print(f"config 5 ({path}) {name}[{b},{h}]: {show(e)}")
    e = check(_np(g["dM"][h]), dM, U.TOL["bf16"], f"config 5 dM ({path})")
    print(f"config 5 ({path}) dM[{h}]: {show(e)}")
