"""Seeded synthetic inputs for DARK attention (numpy only, host side).

This module holds no arithmetic of the method itself: it only draws the
tensors (Q, K, V, M, W, dOut) that both the HIP library and the CPU oracle
consume, in the shapes and value distributions of the five benchmark
configurations.  Anisotropic Gaussians stand in for the query/key statistics of
a pretrained language model, which is the setting the paper argues from
(Section 3: queries and keys share a covariance Lambda that is not a multiple of
the identity).

Recipe
------
* One ``numpy.random.SeedSequence(seed)`` is spawned into seven children used
  in the fixed order U, Q, K, V, M, W, dOut (PCG64 generators).
* Q, K: rows ~ N(0, C_h), C_h = U_h diag(s) U_h^T with U_h a Haar orthogonal
  matrix per head (QR of a Gaussian matrix, sign-fixed); Q and K are independent
  draws sharing C_h.
* V, dOut ~ N(0, 1).  W rows ~ N(0, I_r), one [m, r] block per head.
* M: ``"eye_noise"``: I + 0.1 N(0,1);  ``("cond", kappa)``: U_M diag(sigma)
  V_M^T with sigma log-spaced from 1 down to 1/kappa and Haar U_M, V_M.
* bf16 configurations round Q, K, V, dOut to bfloat16 once (round to nearest
  even) and hand out both the 16-bit patterns and their exact fp32 values.
* ``orthogonal_features``: the other way of drawing W that the paper names
  (Section 2, orthogonal random features): directions orthogonal within blocks
  of r rows, lengths distributed as those of Gaussian vectors.
"""
from __future__ import annotations

from dataclasses import dataclass, field
import numpy as np

__all__ = ["Config", "CONFIGS", "make_inputs", "to_bf16_bits", "bf16_bits_to_f32", "scaled_config",
           "orthogonal_features"]


@dataclass(frozen=True)
class Config:
    name: str
    B: int
    H: int
    L: int
    d: int
    m: int
    dv: int
    dtype: str            # "f32" or "bf16"
    causal: bool
    spectrum: tuple       # ("log", hi, lo) or ("top", k, frac)
    M_kind: tuple         # ("eye_noise", 0.1) or ("cond", kappa)
    chunk: int = 128
    backward: bool = False
    seed: int = 0

    @property
    def r(self) -> int:
        return self.d


CONFIGS = {
    1: Config("cfg1_tiny_bidir_f32", 1, 1, 256, 64, 64, 64, "f32", False, ("log", 10.0, 0.1), ("eye_noise", 0.1)),
    2: Config("cfg2_encoder_bidir_bf16", 8, 12, 4096, 64, 256, 64, "bf16", False, ("log", 100.0, 0.01), ("cond", 10.0)),
    3: Config("cfg3_causal_prefill_bf16", 4, 16, 8192, 128, 256, 128, "bf16", True, ("top", 8, 0.9), ("cond", 20.0)),
    4: Config("cfg4_long_bidir_bf16", 1, 8, 131072, 64, 512, 64, "bf16", False, ("log", 100.0, 0.01), ("cond", 10.0)),
    5: Config("cfg5_finetune_causal_bf16", 2, 12, 4096, 64, 256, 64, "bf16", True, ("log", 100.0, 0.01), ("cond", 10.0),
              backward=True),
}


def scaled_config(cfg: Config, **kw) -> Config:
    """A copy of `cfg` with some fields replaced (smaller parity-test variants)."""
    d = {f: getattr(cfg, f) for f in cfg.__dataclass_fields__}
    d.update(kw)
    return Config(**d)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _haar(rng: np.random.Generator, n: int) -> np.ndarray:
    g = rng.standard_normal((n, n))
    q, rr = np.linalg.qr(g)
    return q * np.sign(np.diag(rr))[None, :]


def _spectrum(cfg: Config) -> np.ndarray:
    d = cfg.d
    kind = cfg.spectrum[0]
    if kind == "log":
        _, hi, lo = cfg.spectrum
        return np.logspace(np.log10(hi), np.log10(lo), d)
    if kind == "top":
        _, k, frac = cfg.spectrum
        total = float(d)
        s = np.empty(d)
        s[:k] = frac * total / k
        s[k:] = (1.0 - frac) * total / (d - k)
        return s
    raise ValueError(kind)


def _make_M(cfg: Config, rng: np.random.Generator) -> np.ndarray:
    H, r, d = cfg.H, cfg.r, cfg.d
    out = np.empty((H, r, d), dtype=np.float32)
    for h in range(H):
        if cfg.M_kind[0] == "eye_noise":
            out[h] = np.eye(r, d) + cfg.M_kind[1] * rng.standard_normal((r, d))
        elif cfg.M_kind[0] == "cond":
            kappa = cfg.M_kind[1]
            sig = np.logspace(0.0, -np.log10(kappa), min(r, d))
            u = _haar(rng, r)
            v = _haar(rng, d)
            out[h] = (u[:, :len(sig)] * sig[None, :]) @ v[:, :len(sig)].T
        elif cfg.M_kind[0] == "eye":
            out[h] = np.eye(r, d)
        else:
            raise ValueError(cfg.M_kind)
    return out


def make_inputs(cfg: Config) -> dict:
    """Draw every tensor of one configuration.

    Returns fp32 arrays "Q","K","V" [B,H,L,*], "M" [H,r,d], "W" [H,m,r] and, for
    backward configurations, "dOut" [B,H,L,dv].  For bf16 configurations the
    fp32 arrays hold exactly the bf16-rounded values and "Q_bits" etc. hold the
    uint16 patterns of the same numbers.
    """
    ss = np.random.SeedSequence(cfg.seed).spawn(7)
    rU, rQ, rK, rV, rM, rW, rG = (np.random.Generator(np.random.PCG64(s)) for s in ss)
    B, H, L, d, m, dv, r = cfg.B, cfg.H, cfg.L, cfg.d, cfg.m, cfg.dv, cfg.r
    s = _spectrum(cfg)
    # T_h = diag(sqrt(s)) U_h^T maps white noise to N(0, U diag(s) U^T).
    T = np.stack([(np.sqrt(s)[:, None] * _haar(rU, d).T) for _ in range(H)]).astype(np.float32)

    def colored(rng):
        x = np.empty((B, H, L, d), dtype=np.float32)
        for b in range(B):
            for h in range(H):
                g = rng.standard_normal((L, d), dtype=np.float32)
                x[b, h] = g @ T[h]
        return x

    out = {"cfg": cfg}
    out["Q"] = colored(rQ)
    out["K"] = colored(rK)
    out["V"] = rV.standard_normal((B, H, L, dv), dtype=np.float32)
    out["M"] = _make_M(cfg, rM)
    out["W"] = rW.standard_normal((H, m, r), dtype=np.float32)
    names = ["Q", "K", "V"]
    if cfg.backward:
        out["dOut"] = rG.standard_normal((B, H, L, dv), dtype=np.float32)
        names.append("dOut")
    if cfg.dtype == "bf16":
        for nme in names:
            bits = to_bf16_bits(out[nme])
            out[nme + "_bits"] = bits
            out[nme] = bf16_bits_to_f32(bits)
    return out


def _gram_schmidt_rows(G: np.ndarray) -> np.ndarray:
    """Orthonormal rows spanning the same nested subspaces as the rows of G (modified Gram-Schmidt,
    each row cleaned twice against the rows before it)."""
    Qm = np.array(G, dtype=np.float64)
    for i in range(Qm.shape[0]):
        for _ in range(2):
            for j in range(i):
                Qm[i] -= (Qm[i] @ Qm[j]) * Qm[j]
        Qm[i] /= np.linalg.norm(Qm[i])
    return Qm


def orthogonal_features(seed: int, H: int, m: int, r: int) -> np.ndarray:
    """W [H, m, r] (fp32) with orthogonal random features (Section 2 of the paper: the directions are
    orthogonalised by Gram-Schmidt; Section 6: the isotropic baseline uses them).

    Per head the m rows come in blocks of r: a block is a Gaussian r x r matrix whose rows are
    orthonormalised, each then given the length of an independent Gaussian vector of r coordinates (a chi
    variable with r degrees of freedom), so that every single row is distributed as N(0, I_r) exactly while
    the rows of a block are mutually orthogonal.  Different blocks, and different heads, are independent.
    """
    root = np.random.SeedSequence(seed)
    W = np.empty((H, m, r), dtype=np.float64)
    for h, child in enumerate(root.spawn(H)):
        rng = np.random.Generator(np.random.PCG64(child))
        for j0 in range(0, m, r):
            Qm = _gram_schmidt_rows(rng.standard_normal((r, r)))
            lengths = np.linalg.norm(rng.standard_normal((r, r)), axis=1)
            n = min(r, m - j0)
            W[h, j0:j0 + n] = (lengths[:, None] * Qm)[:n]
    return W.astype(np.float32)
