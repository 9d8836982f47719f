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


@pytest.mark.parametrize("n,heads", [(2, [(0, 0), (3, 7), (7, 11)]), (4, [(0, 0), (0, 5), (0, 7)])])
def test_bidirectional_configs(n, heads):
    cfg = synth.CONFIGS[n]
    inp = synth.make_inputs(cfg)
    dev = U.to_device(inp, True)
    out = dk.dark_attn_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"])
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
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
    assert bool(torch.isfinite(out).all())
    rows = sorted(set([0, 1, 127, 128, 129, 4095, 4096, 8191] + list(range(5, cfg.L, 97))))
    for b, h in [(0, 0), (1, 3), (2, 9), (3, 15)]:
        want = O.attn_causal(*U.head(inp, b, h), rows=rows)
        e = U.assert_close(_np(out[b, h])[rows], want, U.TOL["bf16"], f"config 3 head {(b, h)}")
        print(f"config 3 head {(b, h)}: {U.fmt(e)}")


@pytest.mark.parametrize("n,heads", [(1, [(0, 0)]), (2, [(0, 0), (5, 3), (7, 11)])])
@pytest.mark.parametrize("is_query", [True, False])
def test_featurize_configs(n, heads, is_query):
    """dark_featurize over the whole Q (query contract) or K (key contract) tensor of configurations 1 and 2,
    through the path DARK_PATH_AUTO picks, against the oracle on sampled (b, h)."""
    cfg = synth.CONFIGS[n]
    bf16 = cfg.dtype == "bf16"
    inp = synth.make_inputs(cfg)
    dev = U.to_device(inp, bf16)
    name = "Q" if is_query else "K"
    phi, stab = dk.dark_featurize(dev[name], dev["M"], dev["W"], is_query)
    torch.cuda.synchronize()
    assert phi.shape == (cfg.B, cfg.H, cfg.L, cfg.m)
    assert bool(torch.isfinite(phi).all()) and bool(torch.isfinite(stab).all())
    tol = U.TOL["bf16" if bf16 else "f32"]
    for b, h in heads:
        W = inp["W"] if inp["W"].ndim == 2 else inp["W"][h]
        want, c = O.featurize(inp[name][b, h], inp["M"][h], W, is_query)
        got_c = _np(stab[b, h]).astype(np.float64)
        # the shift is itself a logit (fp16-rounded operands on the MFMA path)
        assert np.abs(got_c - c).max() <= (2e-2 if bf16 else 1e-4 * max(1.0, np.abs(c).max()))
        # phi * exp(shift difference) is the feature vector under the oracle's shift
        adj = _np(phi[b, h]).astype(np.float64) * np.exp((got_c - c)[:, None] if is_query else (got_c - c))
        e = U.assert_close(adj, want, tol, f"config {n} featurize({name})[{b},{h}]")
        print(f"config {n} featurize({name}) head {(b, h)}: {U.fmt(e)}")


def test_bidirectional_backward_config5_shape():
    """Backward of the bidirectional estimator at the finetuning configuration's shape (fp32 kernels)."""
    cfg = synth.CONFIGS[5]
    inp = synth.make_inputs(cfg)
    dev = U.to_device(inp, True)
    g = dk.dark_attn_bwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], dev["dOut"], False)
    torch.cuda.synchronize()
    for t in g.values():
        assert bool(torch.isfinite(t).all())
    h = 7
    dM = np.zeros((cfg.r, cfg.d))
    for b in range(cfg.B):
        Q, K, V, M, W = U.head(inp, b, h)
        dQ, dK, dV, dMb = O.attn_bwd_brute(Q, K, V, M, W, inp["dOut"][b, h], False)
        dM += dMb
        for name, want in (("dQ", dQ), ("dK", dK), ("dV", dV)):
            e = U.assert_close(_np(g[name][b, h]), want, U.TOL["bf16"], f"bidirectional bwd {name}[{b},{h}]")
            print(f"bidirectional bwd at config 5 shape {name}[{b},{h}]: {U.fmt(e)}")
    e = U.assert_close(_np(g["dM"][h]), dM, U.TOL["bf16"], "bidirectional bwd dM")
    print(f"bidirectional bwd at config 5 shape dM[{h}]: {U.fmt(e)}")


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
