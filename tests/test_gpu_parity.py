"""GPU parity: the HIP library (through the C-ABI binding) against the fp64 oracle,
element by element on the same seeded inputs."""
import ctypes

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


PATHS = [dk.PATH_F32, dk.PATH_AUTO]


# ---------------------------------------------------------------------------
# dark_featurize
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("is_query", [True, False])
def test_featurize(bf16, is_query):
    inp = U.random_problem(1, B=2, H=3, L=150, d=24, r=16, m=80, dv=8, bf16=bf16, amp=3.0)
    dev = U.to_device(inp, bf16)
    phi, stab = dk.dark_featurize(dev["Q"], dev["M"], dev["W"], is_query)
    torch.cuda.synchronize()
    phi, stab = _np(phi), _np(stab)
    tol = U.TOL["bf16" if bf16 else "f32"]
    for b in range(2):
        for h in range(3):
            want, c = O.featurize(inp["Q"][b, h], inp["M"][h], inp["W"][h], is_query)
            got_c = stab[b, h]
            assert np.abs(got_c - c).max() <= 1e-4 * max(1.0, np.abs(c).max())
            U.assert_close(phi[b, h], want, tol, f"phi[{b},{h}]")
            if not bf16:
                # stabiliser-independent comparison in the log domain
                lg = np.log(np.maximum(phi[b, h].astype(np.float64), 1e-300)) + (got_c[:, None] if is_query else got_c)
                ref = O.logits(inp["Q"][b, h], inp["M"][h], inp["W"][h]) - 0.5 * np.log(80)
                big = want > 1e-30            # fp32 features below ~1e-38 flush to zero
                assert np.abs(lg - ref)[big].max() < 2e-4


@pytest.mark.parametrize("is_query", [True, False])
@pytest.mark.parametrize("shape", [(2, 2, 300, 64, 64, 256), (1, 2, 700, 64, 64, 512), (1, 2, 130, 128, 128, 128)])
def test_featurize_fused(shape, is_query):
    """MFMA feature-map kernel (bf16 in and out, fp16 projection operands)."""
    B, H, L, d, r, m = shape
    inp = U.random_problem(3, B=B, H=H, L=L, d=d, r=r, m=m, dv=8, bf16=True, amp=1.5)
    dev = U.to_device(inp, True)
    phi, stab = dk.dark_featurize(dev["Q"], dev["M"], dev["W"], is_query, path=dk.PATH_FUSED)
    torch.cuda.synchronize()
    phi, stab = _np(phi), _np(stab)
    assert np.all(np.isfinite(phi)) and phi.max() <= 1.0 / np.sqrt(m) * (1 + 1e-2)
    for b in range(B):
        for h in range(H):
            want, c = O.featurize(inp["Q"][b, h], inp["M"][h], inp["W"][h], is_query)
            got_c = stab[b, h]
            # the shift is itself a logit computed from fp16-rounded operands
            assert np.abs(got_c - c).max() <= 2e-2
            # phi * exp(shift) is the unstabilised feature vector: compare that, shift-independently
            adj = phi[b, h] * np.exp((got_c - c)[:, None] if is_query else (got_c - c))
            U.assert_close(adj, want, U.TOL["bf16"], f"fused phi[{b},{h}]")


# ---------------------------------------------------------------------------
# M = None: the identity geometry (isotropic positive random features)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("bf16", [False, True])
def test_identity_geometry(bf16, path):
    """Every entry point with M = None against the oracle with M = I (r = d = 64)."""
    inp = U.random_problem(41, 2, 2, 330, 64, 64, 256, 64, bf16=bf16, amp=1.0, backward=True)
    inp["M"] = np.broadcast_to(np.eye(64, dtype=np.float32), (2, 64, 64)).copy()
    dev = U.to_device(inp, bf16)
    tol = U.TOL["bf16" if bf16 else "f32"]
    for causal in (False, True):
        fn = dk.dark_attn_causal_fwd if causal else dk.dark_attn_fwd
        out = fn(dev["Q"], dev["K"], dev["V"], None, dev["W"], path=path)
        torch.cuda.synchronize()
        e = U.assert_close(_np(out), U.oracle_attn(inp, causal), tol, f"M = None, causal={causal}")
        print(f"M = None forward bf16={bf16} path={path} causal={causal}: {U.fmt(e)}")
        g = dk.dark_attn_bwd(dev["Q"], dev["K"], dev["V"], None, dev["W"], dev["dOut"], causal, path=path)
        torch.cuda.synchronize()
        fused_bwd = bf16 and causal and path == dk.PATH_AUTO
        check = U.assert_close_grad if fused_bwd else U.assert_close
        dM = np.zeros((2, 64, 64))
        for b in range(2):
            for h in range(2):
                Q, K, V, M, W = U.head(inp, b, h)
                dQ, dK, dV, dMb = O.attn_bwd_brute(Q, K, V, M, W, inp["dOut"][b, h], causal)
                dM[h] += dMb
                for name, want in (("dQ", dQ), ("dK", dK), ("dV", dV)):
                    check(_np(g[name][b, h]), want, tol, f"M = None, {name}[{b},{h}] causal={causal}")
        check(_np(g["dM"]), dM, tol, f"M = None, dM causal={causal}")
    for is_query in (True, False):
        phi, stab = dk.dark_featurize(dev["Q"], None, dev["W"], is_query, path=path)
        phi2, stab2 = dk.dark_featurize(dev["Q"], dev["M"], dev["W"], is_query, path=path)
        torch.cuda.synchronize()
        assert torch.equal(phi, phi2) and torch.equal(stab, stab2)
    with pytest.raises(dk.DarkError):      # r != d has no identity
        Wr = torch.randn(2, 256, 32, device="cuda")
        p = dk.make_params(2, 2, 330, 64, 32, 256, 64, io_dtype=dk.DARK_BF16 if bf16 else dk.DARK_F32,
                           out_dtype=dk.DARK_BF16 if bf16 else dk.DARK_F32)
        out = torch.empty_like(dev["V"])
        ws = torch.empty(max(dk.workspace_bytes(p, dk.OP_ATTN_FWD), 256), dtype=torch.uint8, device="cuda")
        dk._check(dk.lib().dark_attn_fwd(ctypes.byref(p), dev["Q"].data_ptr(), dev["K"].data_ptr(), dev["V"].data_ptr(),
                                         None, Wr.data_ptr(), out.data_ptr(), ws.data_ptr(), ws.numel(), None), "dark_attn_fwd")


# ---------------------------------------------------------------------------
# dW: the gradient with respect to the draws (learned feature kernel)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("case", ["f32", "bf16_f32path", "bf16_auto", "shared_w", "identity"])
def test_gradient_of_the_draws(case, causal):
    bf16 = case.startswith("bf16") or case == "identity"
    shared = case == "shared_w"
    if case in ("f32", "shared_w"):
        inp = U.random_problem(51, 2, 3, 150, 24, 16, 80, 40, bf16=False, w_shared=shared, amp=2.0, backward=True)
    else:
        inp = U.random_problem(52, 2, 2, 330, 64, 64, 256, 64, bf16=True, amp=1.0, backward=True)
    if case == "identity":
        inp["M"] = np.broadcast_to(np.eye(64, dtype=np.float32), (2, 64, 64)).copy()
    dev = U.to_device(inp, bf16)
    path = dk.PATH_AUTO if case in ("bf16_auto", "identity") else dk.PATH_F32
    g = dk.dark_attn_bwd(dev["Q"], dev["K"], dev["V"], None if case == "identity" else dev["M"], dev["W"], dev["dOut"],
                         causal, path=path, need=("dQ", "dK", "dV", "dM", "dW"))
    g0 = dk.dark_attn_bwd(dev["Q"], dev["K"], dev["V"], None if case == "identity" else dev["M"], dev["W"], dev["dOut"],
                          causal, path=path)
    only = dk.dark_attn_bwd(dev["Q"], dev["K"], dev["V"], None if case == "identity" else dev["M"], dev["W"], dev["dOut"],
                            causal, path=path, need=("dW",))
    torch.cuda.synchronize()
    for k in g0:
        assert torch.equal(g[k], g0[k]), k
    assert torch.equal(only["dW"], g["dW"]) and tuple(g["dW"].shape) == tuple(dev["W"].shape)
    B, H = inp["Q"].shape[:2]
    want = np.zeros(inp["W"].shape)
    for b in range(B):
        for h in range(H):
            Q, K, V, M, W = U.head(inp, b, h)
            dW = O.attn_bwd_brute(Q, K, V, M, W, inp["dOut"][b, h], causal, with_dW=True)[4]
            if shared:
                want += dW
            else:
                want[h] += dW
    fused_bwd = bf16 and causal and path == dk.PATH_AUTO
    check = U.assert_close_grad if fused_bwd else U.assert_close
    tol = U.TOL["bf16"] if bf16 else 2e-4
    e = check(_np(g["dW"]).reshape(-1, want.shape[-1]), want.reshape(-1, want.shape[-1]), tol, f"dW {case} causal={causal}")
    print(f"dW {case} causal={causal}: {(U.fmt_grad if fused_bwd else U.fmt)(e)}")


# ---------------------------------------------------------------------------
# causal forward + backward with the hand-over buffer
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("shape", [(2, 3, 1000, 64, 64, 256, 64), (1, 2, 130, 64, 64, 256, 64), (1, 1, 64, 64, 64, 256, 64)])
def test_saved_state_gives_the_same_bits(shape):
    """dark_attn_causal_fwd_save + dark_attn_bwd_saved against the plain pair: the same kernels on the same
    values, so every output agrees bit for bit; a second, smaller problem through the same buffer as well."""
    B, H, L, d, r, m, dv = shape
    inp = U.random_problem(61, B, H, L, d, r, m, dv, bf16=True, amp=1.5, backward=True)
    dev = U.to_device(inp, True)
    p = dk.make_params(B, H, L, d, r, m, dv, io_dtype=dk.DARK_BF16, out_dtype=dk.DARK_BF16)
    assert dk.saved_bytes(p) > 0
    out0 = dk.dark_attn_causal_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"])
    g0 = dk.dark_attn_bwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], dev["dOut"], True,
                          need=("dQ", "dK", "dV", "dM", "dW"))
    out1, saved = dk.dark_attn_causal_fwd_save(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"])
    assert saved is not None and saved.numel() >= dk.saved_bytes(p)
    # unrelated work through the shared workspace between the two calls must not matter
    dk.dark_attn_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"])
    g1 = dk.dark_attn_bwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], dev["dOut"], True, saved=saved,
                          need=("dQ", "dK", "dV", "dM", "dW"))
    torch.cuda.synchronize()
    assert torch.equal(out0.view(torch.int16), out1.view(torch.int16))
    for k in g0:
        assert torch.equal(g0[k], g1[k]), k
    # errors: a buffer that is too small or missing
    with pytest.raises(dk.DarkError):
        dk.dark_attn_causal_fwd_save(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"],
                                     saved=torch.empty(256, dtype=torch.uint8, device="cuda"))


def test_saved_state_is_a_no_op_where_there_is_no_hand_over():
    """fp32 inputs (fp32 path): dark_saved_bytes is 0, the pair behaves like the plain calls."""
    inp = U.random_problem(62, 1, 2, 200, 24, 16, 80, 40, bf16=False, amp=2.0, backward=True)
    dev = U.to_device(inp, False)
    p = dk.make_params(1, 2, 200, 24, 16, 80, 40)
    assert dk.saved_bytes(p) == 0
    out1, saved = dk.dark_attn_causal_fwd_save(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"])
    assert saved is None
    out0 = dk.dark_attn_causal_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"])
    torch.cuda.synchronize()
    assert torch.equal(out0, out1)


# ---------------------------------------------------------------------------
# forward, small shapes spanning several tiles with ragged tails
# ---------------------------------------------------------------------------
SMALL = [
    # B, H, L,   d,  r,  m,  dv
    (2, 3, 300, 24, 16, 80, 40),
    (1, 2, 257, 64, 64, 64, 64),
    (1, 1, 130, 7, 5, 33, 3),
]


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("shape", SMALL)
@pytest.mark.parametrize("causal", [False, True])
def test_forward_small(shape, bf16, causal, path):
    B, H, L, d, r, m, dv = shape
    inp = U.random_problem(2, B, H, L, d, r, m, dv, bf16=bf16, amp=2.0)
    dev = U.to_device(inp, bf16)
    fn = dk.dark_attn_causal_fwd if causal else dk.dark_attn_fwd
    out = fn(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=path)
    torch.cuda.synchronize()
    want = U.oracle_attn(inp, causal)
    U.assert_close(_np(out), want, U.TOL["bf16" if bf16 else "f32"], f"out {shape} causal={causal}")


# Shapes chosen for the fp32 GEMMs: every tile shape (64, 96 and 128 columns), operands that 16-byte
# loads can fetch and operands they cannot (odd r, m or d), matrix edges inside a group of four
# (dv + 1 = 5, 32, 65, 97 padded to a multiple of four), single rows, and a tile boundary at L.
F32_SWEEP = [
    # B, H, L,   d,  r,  m,   dv
    (1, 1, 1, 4, 4, 4, 4),
    (1, 2, 5, 12, 8, 32, 31),
    (1, 1, 127, 8, 6, 100, 4),
    (1, 1, 128, 64, 64, 256, 64),
    (2, 1, 129, 20, 20, 132, 96),
    (1, 1, 259, 16, 16, 97, 65),
]


@pytest.mark.parametrize("shape", F32_SWEEP)
@pytest.mark.parametrize("causal", [False, True])
def test_f32_path_shape_sweep(shape, causal):
    B, H, L, d, r, m, dv = shape
    inp = U.random_problem(21, B, H, L, d, r, m, dv, amp=1.5)
    dev = U.to_device(inp, False)
    fn = dk.dark_attn_causal_fwd if causal else dk.dark_attn_fwd
    out = fn(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_F32)
    torch.cuda.synchronize()
    U.assert_close(_np(out), U.oracle_attn(inp, causal), U.TOL["f32"], f"fp32 path {shape} causal={causal}")


@pytest.mark.parametrize("chunk", [16, 100, 128, 512])
def test_causal_chunk_is_only_a_schedule(chunk):
    inp = U.random_problem(3, 1, 2, 300, 16, 16, 48, 20)
    dev = U.to_device(inp, False)
    out = dk.dark_attn_causal_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], chunk=chunk)
    torch.cuda.synchronize()
    U.assert_close(_np(out), U.oracle_attn(inp, True), 1e-4, f"chunk={chunk}")


def test_config1_full():
    cfg = synth.CONFIGS[1]
    inp = synth.make_inputs(cfg)
    dev = U.to_device(inp, False)
    out = dk.dark_attn_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"])
    outc = dk.dark_attn_causal_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"])
    torch.cuda.synchronize()
    U.assert_close(_np(out), U.oracle_attn(inp, False), 1e-4, "config 1")
    U.assert_close(_np(outc), U.oracle_attn(inp, True), 1e-4, "config 1 causal")
    # causal and bidirectional agree at the last position
    U.assert_close(_np(outc)[..., -1, :], _np(out)[..., -1, :], 1e-4, "last row")


def test_shared_w_and_scale():
    inp = U.random_problem(4, 2, 2, 96, 16, 8, 40, 12, w_shared=True)
    dev = U.to_device(inp, False)
    out = dk.dark_attn_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], scale=0.2)
    torch.cuda.synchronize()
    U.assert_close(_np(out), U.oracle_attn(inp, False, scale=0.2), 1e-4, "w_shared, scale")


@pytest.mark.parametrize("causal", [False, True])
def test_degenerate_sizes(causal):
    fn = dk.dark_attn_causal_fwd if causal else dk.dark_attn_fwd
    # L = 1, m = 1, d = 1: out == V
    inp = U.random_problem(5, 1, 1, 1, 1, 1, 1, 4)
    dev = U.to_device(inp, False)
    out = fn(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"])
    torch.cuda.synchronize()
    np.testing.assert_allclose(_np(out), inp["V"], rtol=1e-6)
    # empty sequence
    e = {k: v[:, :, :0].contiguous() for k, v in dev.items() if k in ("Q", "K", "V")}
    out = fn(e["Q"], e["K"], e["V"], dev["M"], dev["W"])
    assert out.shape == (1, 1, 0, 4)
    # chunk longer than the sequence
    inp = U.random_problem(6, 1, 1, 40, 8, 8, 16, 4)
    dev = U.to_device(inp, False)
    if causal:
        out = dk.dark_attn_causal_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], chunk=1024)
        torch.cuda.synchronize()
        U.assert_close(_np(out), U.oracle_attn(inp, True), 1e-4, "chunk > L")


def test_large_logits_are_stabilised():
    # logits of several hundred: exp() would overflow fp32 without the stabilising shifts
    # (and logits below -400, which must underflow quietly, as they do in the oracle)
    inp = U.random_problem(7, 1, 1, 200, 16, 16, 32, 8, amp=60.0)
    inp["W"] = inp["W"] * 5.0
    lg = O.logits(inp["K"][0, 0], inp["M"][0], inp["W"][0])
    assert lg.max() > 100 and lg.min() < -400
    dev = U.to_device(inp, False)
    out = dk.dark_attn_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"])
    torch.cuda.synchronize()
    U.assert_close(_np(out), U.oracle_attn(inp, False), 2e-3, "large logits")
    # Causal: the keys of a chunk share one shift per feature, so the spread of one feature's key
    # logits inside a chunk has to fit the fp32 exponent range; a milder case covers that path.
    inp = U.random_problem(7, 1, 1, 200, 16, 16, 32, 8, amp=12.0)
    inp["W"] = inp["W"] * 3.0
    lg = O.logits(inp["K"][0, 0], inp["M"][0], inp["W"][0])
    assert lg.max() > 30 and lg.min() < -60
    dev = U.to_device(inp, False)
    out = dk.dark_attn_causal_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"])
    torch.cuda.synchronize()
    U.assert_close(_np(out), U.oracle_attn(inp, True), 2e-3, "large logits, causal")


def test_bitwise_deterministic():
    inp = U.random_problem(8, 2, 2, 700, 32, 32, 128, 32, bf16=True)
    dev = U.to_device(inp, True)
    for fn in (dk.dark_attn_fwd, dk.dark_attn_causal_fwd):
        a = fn(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"]).clone()
        b = fn(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"])
        torch.cuda.synchronize()
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


# ---------------------------------------------------------------------------
# backward
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", [(2, 2, 200, 24, 16, 48, 20), (1, 1, 130, 16, 16, 64, 16),
                                   (1, 2, 300, 64, 64, 256, 64),   # every GEMM tile shape, ragged
                                   (1, 1, 70, 7, 5, 33, 3)])       # odd sizes: the general GEMM kernel throughout
def test_backward_small(shape, causal, bf16):
    B, H, L, d, r, m, dv = shape
    inp = U.random_problem(9, B, H, L, d, r, m, dv, bf16=bf16, backward=True)
    dev = U.to_device(inp, bf16)
    g = dk.dark_attn_bwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], dev["dOut"], causal, chunk=64,
                         path=dk.PATH_F32)
    torch.cuda.synchronize()
    want = dict(zip(("dQ", "dK", "dV", "dM"), U.oracle_bwd(inp, causal)))
    # gradients are fp32 on both dtypes (inputs only are rounded), so the fp32 path meets the fp32 bar
    tol = 2e-4
    for k in ("dQ", "dK", "dV", "dM"):
        U.assert_close(_np(g[k]), want[k], tol, f"{k} causal={causal}")


FUSED_BWD_SHAPES = [
    # B, H, L
    (1, 2, 300),     # several slices, ragged tail inside the last 32-token tile
    (2, 3, 1000),    # slices of several tiles
    (1, 1, 32),      # exactly one tile
    (1, 1, 7),       # shorter than a tile
    (1, 1, 1),       # a single position: every gradient but dV vanishes
    (1, 1, 2100),    # many slices for one head: long prefix and suffix chains
]


@pytest.mark.parametrize("shape", FUSED_BWD_SHAPES)
def test_fused_backward(shape):
    """MFMA backward (causal, bf16 inputs, d = r = dv = 64, m = 256), forced so that a fall-back cannot pass."""
    B, H, L = shape
    inp = U.random_problem(31, B, H, L, 64, 64, 256, 64, bf16=True, backward=True, amp=2.0)
    dev = U.to_device(inp, True)
    g = dk.dark_attn_bwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], dev["dOut"], True, path=dk.PATH_FUSED)
    torch.cuda.synchronize()
    want = dict(zip(("dQ", "dK", "dV", "dM"), U.oracle_bwd(inp, True)))
    for k in ("dQ", "dK", "dV", "dM"):
        e = U.assert_close_grad(_np(g[k]), want[k], U.TOL["bf16"], f"fused backward {k} {shape}")
        print(f"fused backward {shape} {k}: {U.fmt_grad(e)}")


def test_fused_backward_with_key_logits_rising_far_along_the_sequence():
    """MFMA backward on keys whose logits rise 100 to 200 nats along the sequence (see
    test_causal_key_logits_rising_far_along_the_sequence): the tile kernels work under the running shift of
    their own slice and the suffix sums are rescaled between slices, so the gradients of the first rows, whose
    keys lie ~100 nats below the last slice's shift, are finite and the oracle's."""
    L = 1500
    inp = U.random_problem(38, 1, 1, L, 64, 64, 256, 64, bf16=True, backward=True, amp=1.0)
    inp["K"] = _drifting_keys(inp["K"], 8.0, 38, 6.0)
    _reround(inp, "K")
    assert _first_keys_below_global_shift(inp) > 90.0
    dev = U.to_device(inp, True)
    g = dk.dark_attn_bwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], dev["dOut"], True, path=dk.PATH_FUSED)
    torch.cuda.synchronize()
    want = dict(zip(("dQ", "dK", "dV", "dM"), U.oracle_bwd(inp, True)))
    for k in ("dQ", "dK", "dV", "dM"):
        assert np.isfinite(_np(g[k])).all(), k
        e = U.assert_close_grad(_np(g[k]), want[k], U.TOL["bf16"], f"fused backward, rising key logits, {k}")
        print(f"fused backward, rising key logits, {k}: {U.fmt_grad(e)}")


def test_fused_backward_is_deterministic_and_matches_f32_path():
    inp = U.random_problem(32, 2, 2, 700, 64, 64, 256, 64, bf16=True, backward=True)
    dev = U.to_device(inp, True)
    args = (dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], dev["dOut"], True)
    a = dk.dark_attn_bwd(*args, path=dk.PATH_FUSED)
    a = {k: v.clone() for k, v in a.items()}
    b = dk.dark_attn_bwd(*args, path=dk.PATH_FUSED)
    c = dk.dark_attn_bwd(*args, path=dk.PATH_F32)
    torch.cuda.synchronize()
    for k in ("dQ", "dK", "dV", "dM"):
        assert torch.equal(a[k].view(torch.int32), b[k].view(torch.int32)), k
        U.assert_close_grad(_np(a[k]), _np(c[k]), U.TOL["bf16"], f"fused vs fp32 path, {k}")


def test_backward_optional_outputs():
    inp = U.random_problem(10, 1, 2, 64, 8, 8, 16, 8, backward=True)
    dev = U.to_device(inp, False)
    g = dk.dark_attn_bwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], dev["dOut"], True, need=("dM",))
    torch.cuda.synchronize()
    assert g["dQ"] is None and g["dV"] is None
    U.assert_close(_np(g["dM"]), U.oracle_bwd(inp, True)[3], 2e-4, "dM only")


# ---------------------------------------------------------------------------
# fused MFMA path (bf16 inputs), forced so that a silent fall-back cannot pass
# ---------------------------------------------------------------------------
FUSED_SHAPES = [
    # B, H, L,    d,   r,   m,   dv
    (1, 2, 300, 64, 64, 256, 64),      # ragged tail, several tiles
    (2, 1, 1000, 64, 64, 512, 64),     # two 256-feature blocks
    (1, 1, 64, 64, 64, 256, 64),       # exactly one tile
    (1, 1, 7, 64, 64, 256, 64),        # shorter than a tile
    (1, 2, 333, 128, 128, 256, 128),   # the wide-head instantiation
]


@pytest.mark.parametrize("shape", FUSED_SHAPES)
@pytest.mark.parametrize("out_f32", [False, True])
def test_fused_forward(shape, out_f32):
    B, H, L, d, r, m, dv = shape
    inp = U.random_problem(11, B, H, L, d, r, m, dv, bf16=True, amp=2.0)
    dev = U.to_device(inp, True)
    out = dk.dark_attn_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_FUSED,
                           out_dtype=torch.float32 if out_f32 else None)
    torch.cuda.synchronize()
    assert out.dtype == (torch.float32 if out_f32 else torch.bfloat16)
    e = U.assert_close(_np(out), U.oracle_attn(inp, False), U.TOL["bf16"], f"fused {shape}")
    print(f"fused {shape} out_f32={out_f32}: {U.fmt(e)}")


def test_fused_large_logit_range():
    inp = U.random_problem(12, 1, 1, 500, 64, 64, 256, 64, bf16=True, amp=25.0)
    lg = O.logits(inp["K"][0, 0], inp["M"][0], inp["W"][0])
    assert lg.max() - lg.min() > 100
    dev = U.to_device(inp, True)
    out = dk.dark_attn_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_FUSED)
    torch.cuda.synchronize()
    U.assert_close(_np(out), U.oracle_attn(inp, False), U.TOL["bf16"], "fused, wide logit range")


def _reround(inp, name):
    from paper_2603_04127_amd import synth
    bits = synth.to_bf16_bits(inp[name])
    inp[name + "_bits"] = bits
    inp[name] = synth.bf16_bits_to_f32(bits)


@pytest.mark.parametrize("causal", [False, True])
def test_keys_with_norms_beyond_fp16_range(causal):
    """A few keys so long that their norm term (log2 domain) exceeds what fp16 holds: their features are zero
    to within fp32 next to the ordinary keys, and the result is the oracle's (no clamped norm enters)."""
    inp = U.random_problem(31, 1, 2, 600, 64, 64, 256, 64, bf16=True, amp=1.5)
    rows = [5, 100, 333, 599]
    for h in range(2):
        x = inp["K"][0, h, rows] @ inp["M"][h].T.astype(np.float64)
        inp["K"][0, h, rows] *= (900.0 / np.linalg.norm(x, axis=1))[:, None].astype(np.float32)
    _reround(inp, "K")
    for h in range(2):
        xt = (inp["K"][0, h, rows].astype(np.float64) @ inp["M"][h].T.astype(np.float64)) * 64 ** -0.25
        assert (0.5 * np.log2(np.e) * (xt ** 2).sum(axis=1)).min() > 65504.0
    assert np.abs(inp["K"]).max() < 65504.0
    dev = U.to_device(inp, True)
    fn = dk.dark_attn_causal_fwd if causal else dk.dark_attn_fwd
    out = fn(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"])      # DARK_PATH_AUTO: the MFMA kernels
    ref = fn(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_F32)
    torch.cuda.synchronize()
    want = U.oracle_attn(inp, causal)
    e = U.assert_close(_np(out), want, U.TOL["bf16"], "long keys, auto path")
    U.assert_close(_np(ref), want, U.TOL["bf16"], "long keys, fp32 path")
    print(f"keys beyond the fp16 norm range, causal={causal}: {U.fmt(e)}")


@pytest.mark.parametrize("causal", [False, True])
def test_inputs_beyond_fp16_range_are_not_silently_clamped(causal):
    """bf16 elements above 65504 have no fp16 value: through DARK_PATH_AUTO the affected rows come out
    non-finite (the conversion saturates to infinity), everything else is unaffected; the fp32 kernels
    take such inputs."""
    inp = U.random_problem(32, 1, 3, 300, 64, 64, 256, 64, bf16=True, amp=1.5)
    inp["K"][0, 1, 70, 3] = 1.0e5      # a key of head 1: every later (causal) or every (bidirectional) row of head 1
    inp["Q"][0, 0, 90, 2] = -2.0e5     # a query of head 0: that row only
    _reround(inp, "K")
    _reround(inp, "Q")
    dev = U.to_device(inp, True)
    fn = dk.dark_attn_causal_fwd if causal else dk.dark_attn_fwd
    out = _np(fn(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"]))
    torch.cuda.synchronize()
    want = U.oracle_attn(inp, causal)
    bad_q = ~np.isfinite(out[0, 0]).all(axis=1)
    assert bad_q[90] and bad_q.sum() == 1
    good = np.ones(300, bool)
    good[90] = False
    U.assert_close(out[0, 0][good], want[0, 0][good], U.TOL["bf16"], "head 0, other rows")
    bad_k = ~np.isfinite(out[0, 1]).all(axis=1)
    first = 70 if causal else 0
    assert bad_k[first:].all() and not bad_k[:first].any()
    if causal:
        U.assert_close(out[0, 1][:70], want[0, 1][:70], U.TOL["bf16"], "head 1, rows before the key")
    U.assert_close(out[0, 2], want[0, 2], U.TOL["bf16"], "head 2")
    f32 = _np(fn(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_F32))
    assert np.isfinite(f32).all()


@pytest.mark.parametrize("L", [64, 300, 1100])
def test_fused_rows_with_extreme_logits(L):
    """Queries whose logits spread over hundreds of powers of two (an in-range element of -1000): the readout
    has to take its path with a running row shift, also on the last tile a workgroup handles and on tiles in
    the middle of its run; the row then follows a single feature."""
    inp = U.random_problem(34, 1, 3, L, 64, 64, 256, 64, bf16=True, amp=1.5)
    rows = sorted({0, 17, L // 2, L - 2, L - 1})
    for i, r in enumerate(rows):
        h = i % 3
        for j in range(3 * i, 3 * i + 64):
            # the fp16 operands of the MFMA path carry a logit error of about 2^-11 |w.x~| (a few tenths of
            # a nat here): take a coordinate for which the winning feature leads by a clear margin
            q = inp["Q"][0, h, r].copy()
            q[j % 64] = -1000.0 if i % 2 == 0 else 700.0
            top = np.sort(O.logits(q[None, :], inp["M"][h], inp["W"][h])[0])[-2:]
            if top[1] - top[0] > 12.0:
                inp["Q"][0, h, r] = q
                break
        else:
            raise AssertionError("no coordinate with a clear winner")
    _reround(inp, "Q")
    dev = U.to_device(inp, True)
    for causal in (False, True):
        fn = dk.dark_attn_causal_fwd if causal else dk.dark_attn_fwd
        a = fn(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_FUSED)
        torch.cuda.synchronize()
        e = U.assert_close(_np(a), U.oracle_attn(inp, causal), U.TOL["bf16"], f"extreme rows, L={L} causal={causal}")
        print(f"rows with extreme logits L={L} causal={causal}: {U.fmt(e)}")


@pytest.mark.parametrize("scale", [1e-6, 1e-3, 4.0])
def test_fused_matches_f32_path_at_extreme_amplitudes(scale):
    """Tiny inputs (fp16 subnormals and below: the logits are ~0 either way) and large ones (logits spread
    over about 180 nats)."""
    inp = U.random_problem(33, 1, 2, 400, 64, 64, 256, 64, bf16=True, amp=1.0)
    for n in ("Q", "K"):
        inp[n] *= np.float32(scale)
        _reround(inp, n)
    dev = U.to_device(inp, True)
    for causal in (False, True):
        fn = dk.dark_attn_causal_fwd if causal else dk.dark_attn_fwd
        a = fn(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_FUSED)
        c = fn(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_F32)
        torch.cuda.synchronize()
        want = U.oracle_attn(inp, causal)
        e = U.assert_close(_np(a), want, U.TOL["bf16"], f"fused, inputs x{scale}")
        U.assert_close(_np(c), want, U.TOL["bf16"], f"fp32 path, inputs x{scale}")
        print(f"inputs x{scale} causal={causal}: fused {U.fmt(e)}")


@pytest.mark.parametrize("causal", [False, True])
def test_logit_spread_beyond_the_supported_range(causal):
    """Inputs 15 times the usual size: key logits spread over ~1900 nats along the sequence, far beyond the
    ~80 nats the kernels with one shift per (b, h) (MFMA paths: one scalar per running prefix or feature
    block) are specified for.  The MFMA paths then return non-finite rows (0/0) where every key a row depends
    on has vanished below the shift, and since all features share that shift, whatever survives dominates
    what vanished: the finite rows are still the oracle's.  The bidirectional fp32 kernels have no such
    limit.  (The fp32 causal kernels keep their shifts per chunk and are specified for a spread of ~80 nats
    inside a chunk, which this input exceeds many times over; they are not checked here.)"""
    inp = U.random_problem(33, 1, 2, 400, 64, 64, 256, 64, bf16=True, amp=1.0)
    for n in ("Q", "K"):
        inp[n] *= np.float32(15.0)
        _reround(inp, n)
    dev = U.to_device(inp, True)
    fn = dk.dark_attn_causal_fwd if causal else dk.dark_attn_fwd
    want = U.oracle_attn(inp, causal)
    for path, name in ((dk.PATH_FUSED, "fused"), (dk.PATH_F32, "f32")):
        if causal and name == "f32":
            continue
        got = _np(fn(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=path))
        torch.cuda.synchronize()
        finite = np.isfinite(got).all(axis=-1)
        if name == "f32":
            assert finite.all()
        assert finite.mean() > 0.5
        # the MFMA path's fp16 operands carry a logit error that grows with the logits (2^-11 |w.x~|)
        tol = 1.5 * U.TOL["bf16"] if name == "fused" else U.TOL["bf16"]
        e = U.assert_close(got[finite], want[finite], tol, f"x15 inputs, {name}, causal={causal}")
        print(f"x15 inputs {name} causal={causal}: {int((~finite).sum())} of {finite.size} rows non-finite; finite rows: {U.fmt(e)}")


@pytest.mark.parametrize("path", PATHS)
def test_causal_key_logits_growing_along_the_sequence(path):
    """Keys whose norm shrinks along the sequence, so that the key logits rise by about 60 nats from the
    first token to the last (inside the ~80 nats the causal kernels are specified for): early rows see only
    keys far below the shift that later keys set."""
    inp = U.random_problem(35, 1, 2, 700, 64, 64, 256, 64, bf16=True, amp=1.0)
    ramp = np.linspace(5.0, 1.0, 700, dtype=np.float32)[None, None, :, None]
    inp["K"] = inp["K"] * ramp
    _reround(inp, "K")
    lg = O.logits(inp["K"][0, 0], inp["M"][0], inp["W"][0]).max(axis=1)
    assert 40.0 < lg[-50:].mean() - lg[:50].mean() < 80.0
    dev = U.to_device(inp, True)
    got = _np(dk.dark_attn_causal_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=path))
    torch.cuda.synchronize()
    e = U.assert_close(got, U.oracle_attn(inp, True), U.TOL["bf16"], f"rising key logits, {path}")
    print(f"causal, key logits rising ~60 nats along the sequence ({path}): {U.fmt(e)}")


def _drifting_keys(K, r0, seed, elen):
    """Keys = a fixed direction of length elen times a factor that falls from r0 to 1 along the sequence, plus
    0.3 of the given keys: every feature's key logits rise smoothly along the sequence (through the norm term)
    while neighbouring keys stay within a few nats of each other."""
    B, H, L, d = K.shape
    e = np.random.default_rng(seed).standard_normal((1, H, 1, d))
    e = elen * e / np.linalg.norm(e, axis=-1, keepdims=True)
    ramp = np.linspace(r0, 1.0, L)[None, None, :, None]
    return (ramp * e + 0.3 * K).astype(np.float32)


def _first_keys_below_global_shift(inp):
    """Smallest distance, over the features, between a feature's largest key logit of the whole sequence and
    its largest over the first ten keys (head 0)."""
    lg = O.logits(inp["K"][0, 0], inp["M"][0], inp["W"][0])
    return float((lg.max(axis=0) - lg[:10].max(axis=0)).min())


@pytest.mark.parametrize("path", PATHS)
def test_causal_key_logits_rising_far_along_the_sequence(path):
    """Every feature's key logits rise by 100 to 200 nats from the first token to the last: under one shift
    per feature for the whole sequence all features of the first keys would underflow fp32 (e^-88) and the
    first rows would be 0/0.  The causal kernels keep their shifts per chunk (fp32 kernels: running maxima
    per feature, the chunk states rescaled where they are added up) or per slice (MFMA kernels: a running
    scalar), so only the spread inside a chunk or slice counts (here about 30 nats)."""
    L = 2000
    inp = U.random_problem(36, 1, 2, L, 64, 64, 256, 64, bf16=True, amp=1.0)
    inp["K"] = _drifting_keys(inp["K"], 8.0, 36, 6.0)
    _reround(inp, "K")
    gap = _first_keys_below_global_shift(inp)
    assert gap > 90.0
    dev = U.to_device(inp, True)
    got = _np(dk.dark_attn_causal_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=path))
    torch.cuda.synchronize()
    assert np.isfinite(got).all()
    e = U.assert_close(got, U.oracle_attn(inp, True), U.TOL["bf16"], f"key logits rising far, {path}")
    print(f"causal, first keys {gap:.0f} nats below every feature's largest key logit ({path}): {U.fmt(e)}")


def test_causal_backward_with_key_logits_rising_far_along_the_sequence():
    """Gradients of the fp32 causal kernels on the same kind of input: the suffix sums of the backward are
    rescaled between chunks like the prefix sums of the forward."""
    L = 600
    inp = U.random_problem(37, 1, 1, L, 16, 16, 64, 16, amp=1.0)
    inp["K"] = _drifting_keys(inp["K"], 8.0, 37, 4.0)
    assert _first_keys_below_global_shift(inp) > 88.0
    rng = np.random.default_rng(5)
    G = rng.standard_normal(inp["V"].shape).astype(np.float32)
    dev = U.to_device(inp, False)
    g = dk.dark_attn_bwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], torch.from_numpy(G).cuda(), True, chunk=64)
    torch.cuda.synchronize()
    want = O.attn_bwd_brute(inp["Q"][0, 0], inp["K"][0, 0], inp["V"][0, 0], inp["M"][0], inp["W"][0], G[0, 0], True)
    for name, w in zip(("dQ", "dK", "dV", "dM"), want):
        got = _np(g[name])
        got = got[0, 0] if name != "dM" else got[0]
        assert np.isfinite(got).all(), name
        U.assert_close_grad(got, w, 2e-4, f"rising key logits, {name}")


def test_fused_matches_f32_path_and_is_deterministic():
    inp = U.random_problem(13, 2, 3, 900, 64, 64, 256, 64, bf16=True)
    dev = U.to_device(inp, True)
    a = dk.dark_attn_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_FUSED).clone()
    b = dk.dark_attn_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_FUSED)
    c = dk.dark_attn_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_F32)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    U.assert_close(_np(a), _np(c), U.TOL["bf16"], "fused vs fp32 path")


@pytest.mark.parametrize("L,wgs", [(1000, 2), (1000, 6), (4096 + 37, 2), (200, 2)])
def test_fused_long_slices(L, wgs):
    """Few workgroups in the key/value pass, so that one slice runs over many tiles (the small shapes
    above give every workgroup one or two): the pass's buffers rotate several times, with a ragged last
    tile."""
    inp = U.random_problem(21, 1, 2, L, 64, 64, 256, 64, bf16=True, amp=2.0)
    dev = U.to_device(inp, True)
    out = dk.dark_attn_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_FUSED, sched={"kv_wgs": wgs})
    torch.cuda.synchronize()
    e = U.assert_close(_np(out), U.oracle_attn(inp, False), U.TOL["bf16"], f"fused long slices L={L} wgs={wgs}")
    print(f"fused long slices L={L} wgs={wgs}: {U.fmt(e)}")


def test_fused_shift_raised_mid_slice():
    """Keys ordered by growing norm inside one long slice: the per-feature shifts chosen from the first
    block are far too low for the later ones, so the rare path (raise the shift, rescale the state) runs
    in the middle of the slice."""
    inp = U.random_problem(22, 1, 1, 900, 64, 64, 256, 64, bf16=True, amp=1.0)
    ramp = np.linspace(0.02, 8.0, 900, dtype=np.float32)[None, None, :, None]
    from paper_2603_04127_amd import synth
    bits = synth.to_bf16_bits(inp["K"] * ramp)
    inp["K_bits"], inp["K"] = bits, synth.bf16_bits_to_f32(bits)
    inp["W"] = inp["W"] * 3.0  # a key logit is at most |w_j|^2 / 2: longer draws leave room above the first block
    lg = O.logits(inp["K"][0, 0], inp["M"][0], inp["W"][0])
    first, later = lg[:32].max(axis=0), lg[32:].max(axis=0)
    # 2^40 = 27.7 nats above the first block's shift is where the kernel raises a feature's shift
    assert np.sum(later - first > 30.0) > 50
    dev = U.to_device(inp, True)
    out = dk.dark_attn_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_FUSED, sched={"kv_wgs": 1})
    torch.cuda.synchronize()
    U.assert_close(_np(out), U.oracle_attn(inp, False), U.TOL["bf16"], "fused, shift raised mid-slice")


def test_fused_exponential_overflows_mid_slice():
    """A steeper ramp: from one 32-token block to the next some key logits rise by more than 2^128 = 88.7 nats,
    so that under the shift in force the exponential itself overflows.  The key pass sees that only after the
    block, in the running sum z, and has to redo the block under a raised shift before anything of it reaches
    the state."""
    from paper_2603_04127_amd import synth
    inp = U.random_problem(22, 1, 1, 900, 64, 64, 256, 64, bf16=True, amp=1.0)
    ramp = np.linspace(0.02, 10.0, 900, dtype=np.float32)[None, None, :, None]
    bits = synth.to_bf16_bits(inp["K"] * ramp)
    inp["K_bits"], inp["K"] = bits, synth.bf16_bits_to_f32(bits)
    inp["W"] = inp["W"] * 5.0
    lg = O.logits(inp["K"][0, 0], inp["M"][0], inp["W"][0])
    run, jump = lg[:32].max(axis=0), np.zeros(lg.shape[1])
    for b in range(1, (900 + 31) // 32):
        bm = lg[32 * b:32 * b + 32].max(axis=0)
        jump, run = np.maximum(jump, bm - run), np.maximum(run, bm)
    # (the shift in force is at most the running maximum, so the rise the kernel sees is at least this one)
    assert np.sum(jump > 95.0) >= 2, np.sort(jump)[-8:]
    dev = U.to_device(inp, True)
    out = dk.dark_attn_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_FUSED, sched={"kv_wgs": 1})
    torch.cuda.synchronize()
    U.assert_close(_np(out), U.oracle_attn(inp, False), U.TOL["bf16"], "fused, exponential overflows mid-slice")


# ---------------------------------------------------------------------------
# fused MFMA causal path (bf16 inputs), forced
# ---------------------------------------------------------------------------
FUSED_CAUSAL_SHAPES = [
    # B, H, L,    d,   r,   m,   dv
    (1, 2, 300, 64, 64, 256, 64),      # several slices, ragged tail inside the last tile
    (2, 3, 1000, 64, 64, 256, 64),     # slices of more than one key tile
    (1, 1, 32, 64, 64, 256, 64),       # exactly one scan tile
    (1, 1, 7, 64, 64, 256, 64),        # shorter than a tile
    (1, 1, 1, 64, 64, 256, 64),        # a single position: out == v
    (1, 1, 2100, 64, 64, 256, 64),     # many slices for one head: long prefix chain
    (1, 2, 333, 128, 128, 256, 128),   # wide head: the state waves own two blocks of value columns each
    (2, 2, 900, 128, 128, 256, 128),
]


@pytest.mark.parametrize("shape", FUSED_CAUSAL_SHAPES)
@pytest.mark.parametrize("out_f32", [False, True])
def test_fused_causal_forward(shape, out_f32):
    B, H, L, d, r, m, dv = shape
    inp = U.random_problem(21, B, H, L, d, r, m, dv, bf16=True, amp=2.0)
    dev = U.to_device(inp, True)
    out = dk.dark_attn_causal_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_FUSED,
                                  out_dtype=torch.float32 if out_f32 else None)
    torch.cuda.synchronize()
    assert out.dtype == (torch.float32 if out_f32 else torch.bfloat16)
    e = U.assert_close(_np(out), U.oracle_attn(inp, True), U.TOL["bf16"], f"fused causal {shape}")
    print(f"fused causal {shape} out_f32={out_f32}: {U.fmt(e)}")


@pytest.mark.parametrize("L,d,wgs", [(1000, 64, 2), (4096 + 37, 64, 2), (777, 128, 2), (33, 128, 1), (65, 64, 1)])
def test_fused_causal_long_slices(L, d, wgs):
    """Few workgroups in the causal pass, so that one slice runs over many tiles: the scan's feature waves run a
    tile ahead of its state waves through double-buffered patches many times over, with a ragged last tile
    (and, for the shortest cases, a last tile of one token right after the first)."""
    inp = U.random_problem(25, 1, 2, L, d, d, 256, d, bf16=True, amp=2.0)
    dev = U.to_device(inp, True)
    out = dk.dark_attn_causal_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_FUSED,
                                  sched={"cs_wgs": wgs})
    torch.cuda.synchronize()
    e = U.assert_close(_np(out), U.oracle_attn(inp, True), U.TOL["bf16"], f"fused causal long slices L={L} d={d}")
    print(f"fused causal long slices L={L} d={d} wgs={wgs}: {U.fmt(e)}")


def test_fused_causal_first_row_and_last_row():
    inp = U.random_problem(22, 1, 2, 500, 64, 64, 256, 64, bf16=True)
    dev = U.to_device(inp, True)
    c = dk.dark_attn_causal_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_FUSED,
                                out_dtype=torch.float32)
    b = dk.dark_attn_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_FUSED,
                         out_dtype=torch.float32)
    torch.cuda.synchronize()
    # position 0 sees only itself; the last position sees everything (bidirectional result)
    np.testing.assert_allclose(_np(c)[:, :, 0], inp["V"][:, :, 0], rtol=1e-5, atol=1e-5)
    U.assert_close(_np(c)[:, :, -1], _np(b)[:, :, -1], U.TOL["bf16"], "last row")


def test_fused_causal_matches_f32_path_and_is_deterministic():
    inp = U.random_problem(23, 2, 3, 900, 64, 64, 256, 64, bf16=True)
    dev = U.to_device(inp, True)
    a = dk.dark_attn_causal_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_FUSED).clone()
    b = dk.dark_attn_causal_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_FUSED)
    c = dk.dark_attn_causal_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_F32)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    U.assert_close(_np(a), _np(c), U.TOL["bf16"], "fused causal vs fp32 path")


def test_fused_causal_wide_logit_range():
    inp = U.random_problem(24, 1, 1, 700, 64, 64, 256, 64, bf16=True, amp=8.0)
    lg = O.logits(inp["K"][0, 0], inp["M"][0], inp["W"][0])
    assert lg.max() - lg.min() > 40
    dev = U.to_device(inp, True)
    out = dk.dark_attn_causal_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], path=dk.PATH_FUSED)
    torch.cuda.synchronize()
    U.assert_close(_np(out), U.oracle_attn(inp, True), U.TOL["bf16"], "fused causal, wide logit range")
