"""Self-tests of the seeded input generators (no method arithmetic involved)."""
import numpy as np
import torch

from paper_2603_04127_amd import synth


def test_bf16_rounding_matches_torch():
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32) * 37.0
    bits = synth.to_bf16_bits(x)
    t = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(bits.view(np.int16), t.view(torch.int16).numpy())
    assert np.array_equal(synth.bf16_bits_to_f32(bits), t.float().numpy())


def test_config_table_matches_benchmark_shapes():
    c = synth.CONFIGS
    assert (c[1].B, c[1].H, c[1].L, c[1].d, c[1].m, c[1].dv, c[1].dtype) == (1, 1, 256, 64, 64, 64, "f32")
    assert (c[2].B, c[2].H, c[2].L, c[2].d, c[2].m, c[2].dv, c[2].dtype) == (8, 12, 4096, 64, 256, 64, "bf16")
    assert (c[3].B, c[3].H, c[3].L, c[3].d, c[3].m, c[3].dv, c[3].causal, c[3].chunk) == (4, 16, 8192, 128, 256, 128, True, 128)
    assert (c[4].B, c[4].H, c[4].L, c[4].d, c[4].m, c[4].dv) == (1, 8, 131072, 64, 512, 64)
    assert (c[5].B, c[5].H, c[5].L, c[5].d, c[5].m, c[5].dv, c[5].backward, c[5].causal) == (2, 12, 4096, 64, 256, 64, True, True)


def test_seeded_and_distribution():
    cfg = synth.scaled_config(synth.CONFIGS[2], B=1, H=2, L=8192)
    a = synth.make_inputs(cfg)
    b = synth.make_inputs(cfg)
    for k in ("Q", "K", "V", "M", "W"):
        assert np.array_equal(a[k], b[k])
    # covariance spectrum of the rows of Q (log-spaced 100 .. 0.01, bf16-rounded draws)
    q = a["Q"][0, 0].astype(np.float64)
    ev = np.sort(np.linalg.eigvalsh(q.T @ q / q.shape[0]))[::-1]
    want = np.logspace(2, -2, cfg.d)
    assert np.all(np.abs(np.log(ev / want)) < 0.25)
    # Q and K share the covariance but are independent draws
    k = a["K"][0, 0].astype(np.float64)
    assert abs(np.trace(k.T @ k) / np.trace(q.T @ q) - 1) < 0.1 and not np.array_equal(q, k)
    # M: singular values log-spaced 1 .. 1/kappa, a different matrix per head
    sv = np.linalg.svd(a["M"][0].astype(np.float64), compute_uv=False)
    np.testing.assert_allclose(sv, np.logspace(0, -1, cfg.d), rtol=1e-4)
    assert not np.allclose(a["M"][0], a["M"][1])
    assert abs(a["W"].std() - 1) < 0.02 and abs(a["V"].std() - 1) < 0.02
    assert np.array_equal(synth.bf16_bits_to_f32(a["Q_bits"]), a["Q"])


def test_top_k_spectrum():
    cfg = synth.scaled_config(synth.CONFIGS[3], B=1, H=1, L=16384)
    q = synth.make_inputs(cfg)["Q"][0, 0].astype(np.float64)
    ev = np.sort(np.linalg.eigvalsh(q.T @ q / q.shape[0]))[::-1]
    assert abs(ev[:8].sum() / ev.sum() - 0.9) < 0.01
    assert abs(ev.sum() / cfg.d - 1) < 0.05


# --- orthogonal random features (Section 2 of the paper: Gram-Schmidt orthogonalised directions) -------------
def test_orthogonal_features_blocks_are_orthogonal_with_gaussian_lengths():
    import scipy.stats
    H, m, r = 5, 200, 32
    W32 = synth.orthogonal_features(3, H, m, r)
    assert W32.shape == (H, m, r) and W32.dtype == np.float32
    W = W32.astype(np.float64)
    assert np.array_equal(synth.orthogonal_features(3, H, m, r), synth.orthogonal_features(3, H, m, r))
    assert not np.array_equal(synth.orthogonal_features(3, H, m, r), synth.orthogonal_features(4, H, m, r))
    for h in range(H):
        for j0 in range(0, m, r):
            blk = W[h, j0:j0 + r]                      # the last block is ragged (200 = 6 * 32 + 8)
            n = np.linalg.norm(blk, axis=1)
            G = (blk / n[:, None]) @ (blk / n[:, None]).T
            assert np.abs(G - np.eye(len(blk))).max() < 1e-6      # fp32 storage of the rows
        # rows of different blocks are independent draws: not orthogonal
        assert np.abs(W[h, :r] @ W[h, r:2 * r].T).max() > 1.0
    # every single row is N(0, I_r): its length is chi(r), its coordinates standard normal
    lengths = np.linalg.norm(W.reshape(-1, r), axis=1)
    assert scipy.stats.kstest(lengths, "chi", args=(r,)).pvalue > 1e-3
    assert scipy.stats.kstest(W.ravel(), "norm").pvalue > 1e-3
    # fewer rows than one block, and a head count of one
    assert synth.orthogonal_features(0, 1, 5, 16).shape == (1, 5, 16)
