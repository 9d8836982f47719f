"""dark_whiten (Section 4.1, Proposition C.1: M = Lambda^{-1/2}) against the fp64 oracle.

The rows of M are determined up to sign (and up to rotations inside nearly equal eigenvalues), so what is
compared is what is unique: the covariance estimate, Sigma = M^T M, and the whitening property
M Lambda M^T = I_r with the oracle's Lambda."""
import numpy as np
import pytest

import paper_2603_04127_amd as dk
from paper_2603_04127_amd import synth
from oracle import dark_oracle as O
from tests import parity_util as U

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _np(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def _check_head(Mg, covg, Qh, Kh, r, what, tol_cov=2e-5, tol=5e-3):
    """Qh, Kh: [B, L, d] rows of one head (Kh may be None)."""
    d = Qh.shape[-1]
    rows_q = Qh.reshape(-1, d)
    rows_k = rows_q[:0] if Kh is None else Kh.reshape(-1, d)
    Mo, Lam = O.whitening_geometry(rows_q, rows_k, r=r)
    assert np.abs(covg - Lam).max() <= tol_cov * np.abs(Lam).max(), what + ": covariance"
    W = Mg @ Lam @ Mg.T
    e_white = np.abs(W - np.eye(r)).max()
    Sg, So = Mg.T @ Mg, Mo.T @ Mo
    e_sigma = np.abs(Sg - So).max() / np.abs(So).max()
    print(f"{what}: |cov - Lambda| / max {np.abs(covg - Lam).max() / np.abs(Lam).max():.2e}, "
          f"|M Lambda M^T - I| {e_white:.2e}, |Sigma - Sigma_oracle| / max {e_sigma:.2e}, "
          f"condition number {np.linalg.cond(Lam):.1e}")
    assert e_white <= tol and e_sigma <= tol, what


@pytest.mark.parametrize("shape", [
    # B, H, L,    d,   r,   bf16
    (2, 3, 700,   24,  24,  False),
    (1, 2, 2500,  24,  10,  False),
    (3, 2, 300,   7,   7,   False),     # odd d: the rotation schedule plays against a dummy index
    (2, 2, 5000,  64,  64,  True),      # MFMA moments, several chunks per sequence, ragged tile
    (1, 2, 1000,  128, 128, True),
    (1, 2, 900,   128, 32,  True),
    (2, 2, 640,   40,  40,  True),      # bf16 without the MFMA kernel
])
def test_whiten_small(shape):
    B, H, L, d, r, bf16 = shape
    inp = U.random_problem(71, B, H, L, d, d, 16, 8, bf16=bf16, amp=1.5)
    inp["Q"] = inp["Q"] + np.float32(0.3)      # a non-zero mean: the covariance is centred
    inp["K"] = inp["K"] + np.float32(0.3)
    if bf16:
        for n in ("Q", "K"):
            bits = synth.to_bf16_bits(inp[n])
            inp[n + "_bits"] = bits
            inp[n] = synth.bf16_bits_to_f32(bits)
    dev = U.to_device(inp, bf16)
    M, cov = dk.dark_whiten(dev["Q"], dev["K"], r=r, want_cov=True)
    M2 = dk.dark_whiten(dev["Q"], dev["K"], r=r)
    torch.cuda.synchronize()
    assert tuple(M.shape) == (H, r, d) and torch.equal(M, M2)        # deterministic, cov_out optional
    assert bool(torch.isfinite(M).all())
    for h in range(H):
        _check_head(_np(M[h]), _np(cov[h]), inp["Q"][:, h].astype(np.float64), inp["K"][:, h].astype(np.float64), r,
                    f"whiten {shape} head {h}")


def test_whiten_queries_only_and_degenerate_direction():
    inp = U.random_problem(72, 2, 2, 800, 24, 24, 16, 8, bf16=False, amp=1.0)
    inp["Q"][..., 5] = 2.0          # a coordinate without variance: its eigenvalue is floored, M stays finite
    dev = U.to_device(inp, False)
    M, cov = dk.dark_whiten(dev["Q"], None, want_cov=True)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(M).all())
    for h in range(2):
        Mo, Lam = O.whitening_geometry(inp["Q"][:, h].reshape(-1, 24).astype(np.float64), np.zeros((0, 24)))
        assert np.abs(_np(cov[h]) - Lam).max() <= 2e-5 * np.abs(Lam).max()
        lam = np.linalg.eigvalsh(Lam)
        # on the 23 directions that carry variance the geometry is the oracle's
        P = np.eye(24)
        P = np.delete(P, 5, axis=0)
        Sg, So = P @ _np(M[h]).T @ _np(M[h]) @ P.T, P @ Mo.T @ Mo @ P.T
        assert np.abs(Sg - So).max() <= 5e-3 * np.abs(So).max()
        assert np.abs(_np(M[h])).max() <= 1.01 / np.sqrt(1e-6 * lam.max())


def test_whiten_rejects_what_it_does_not_take():
    q = torch.zeros(1, 1, 64, 256, device="cuda")
    with pytest.raises(dk.DarkError):
        dk.dark_whiten(q, q)            # d > 128
    q = torch.zeros(1, 1, 64, 16, device="cuda")
    with pytest.raises(dk.DarkError):
        dk.dark_whiten(q, q, r=17)      # r > d


@pytest.mark.parametrize("n,heads", [(2, [0, 7]), (3, [3])])
def test_whiten_configs(n, heads):
    """Whole Q, K of configurations 2 (condition number 1e4) and 3, oracle on sampled heads."""
    cfg = synth.CONFIGS[n]
    inp = synth.make_inputs(cfg)
    dev = U.to_device(inp, True)
    M, cov = dk.dark_whiten(dev["Q"], dev["K"], want_cov=True)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(M).all())
    for h in heads:
        _check_head(_np(M[h]), _np(cov[h]), inp["Q"][:, h].astype(np.float64), inp["K"][:, h].astype(np.float64), cfg.d,
                    f"whiten config {n} head {h}", tol=2e-2)
