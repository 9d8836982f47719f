"""dark_decode_step: the causal recurrence one token at a time against the oracle's causal attention."""
import numpy as np
import pytest

import paper_2603_04127_amd as dk
from oracle import dark_oracle as O
from tests import parity_util as U

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _np(t):
    return t.detach().float().cpu().numpy()


@pytest.mark.parametrize("shape", [
    # B, H, L,  d,  r,  m,   dv, bf16, shared W, identity
    (2, 3, 70, 24, 16, 80,  40, False, False, False),   # a thread per column
    (1, 2, 50, 7,  5,  33,  3,  False, False, False),
    (2, 2, 90, 64, 64, 256, 64, True,  False, False),   # 16-byte state accesses
    (1, 2, 40, 64, 64, 256, 64, True,  True,  False),
    (1, 2, 40, 32, 32, 64,  16, False, False, True),
])
def test_decode_matches_causal_attention(shape):
    B, H, L, d, r, m, dv, bf16, shared, ident = shape
    inp = U.random_problem(81, B, H, L, d, r, m, dv, bf16=bf16, w_shared=shared, amp=2.0)
    if ident:
        inp["M"] = np.broadcast_to(np.eye(d, dtype=np.float32), (H, d, d)).copy()
    dev = U.to_device(inp, bf16)
    state = dk.decode_state(B, H, m, dv)
    outs = []
    for t in range(L):
        outs.append(dk.dark_decode_step(dev["Q"][:, :, t].contiguous(), dev["K"][:, :, t].contiguous(),
                                        dev["V"][:, :, t].contiguous(), None if ident else dev["M"], dev["W"], state))
    torch.cuda.synchronize()
    got = _np(torch.stack(outs, dim=2))
    want = U.oracle_attn(inp, True)
    e = U.assert_close(got, want, U.TOL["bf16" if bf16 else "f32"], f"decode {shape}")
    print(f"decode {shape}: {U.fmt(e)}")
    # the state is the causal state: z = sum_l phi(k_l) under the stored shift
    S, z, c = state
    for b in range(B):
        for h in range(H):
            Q, K, V, M, W = U.head(inp, b, h)
            lg = O.logits(K, M, W)
            zw = np.exp(lg - float(c[b, h])).sum(0)
            assert abs(float(c[b, h]) - lg.max()) <= 1e-3 * max(1.0, abs(lg.max()))
            assert np.abs(_np(z[b, h]) - zw).max() <= 2e-3 * zw.max()


def test_decode_rescales_when_the_key_logits_rise():
    """Keys whose logits grow by tens of nats from token to token: every step raises the shift."""
    inp = U.random_problem(82, 1, 2, 60, 24, 16, 80, 40, bf16=False, amp=1.0)
    ramp = np.linspace(4.0, 0.5, 60, dtype=np.float32)[None, None, :, None]
    inp["K"] = inp["K"] * ramp
    dev = U.to_device(inp, False)
    state = dk.decode_state(1, 2, 80, 40)
    outs = [dk.dark_decode_step(dev["Q"][:, :, t].contiguous(), dev["K"][:, :, t].contiguous(),
                                dev["V"][:, :, t].contiguous(), dev["M"], dev["W"], state) for t in range(60)]
    torch.cuda.synchronize()
    U.assert_close(_np(torch.stack(outs, dim=2)), U.oracle_attn(inp, True), U.TOL["f32"], "decode, rising logits")
