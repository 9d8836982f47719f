"""dark_attn_fwd_static (the entry point that allocates nothing) against dark_attn_fwd, through the
C ABI: two calls in a row on the static scratch, the second with a smaller input, must each give what
dark_attn_fwd gives on a caller-owned workspace (same kernels, same schedule: bitwise), and both must
match the oracle to the forward bar."""
import numpy as np
import pytest

import paper_2603_04127_amd as dk
from tests import parity_util as U

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _np(t):
    return t.detach().float().cpu().numpy()


@pytest.mark.parametrize("bf16,shapes", [
    (True, [(2, 3, 1500, 64, 64, 256, 64), (1, 2, 300, 64, 64, 256, 64)]),      # fused MFMA kernels
    (False, [(1, 2, 700, 24, 16, 80, 40), (1, 1, 130, 24, 16, 80, 40)]),        # fp32 kernels
])
def test_static_scratch_matches_workspace_entry_point(bf16, shapes):
    assert dk.static_scratch_bytes() == 32 * 1024 * 1024
    for k, shape in enumerate(shapes):   # the second call reuses the array the first one left behind
        B, H, L, d, r, m, dv = shape
        inp = U.random_problem(31 + k, B, H, L, d, r, m, dv, bf16=bf16, amp=2.0)
        dev = U.to_device(inp, bf16)
        ref = dk.dark_attn_fwd(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"])
        out = torch.full_like(ref, float("nan"))
        torch.cuda.synchronize()
        dk.dark_attn_fwd_static(dev["Q"], dev["K"], dev["V"], dev["M"], dev["W"], out)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16 if bf16 else torch.int32), ref.view(torch.int16 if bf16 else torch.int32))
        U.assert_close(_np(out), U.oracle_attn(inp, False), U.TOL["bf16" if bf16 else "f32"], f"static {shape}")


def test_static_scratch_rejects_oversized_problem():
    # config-4-sized problem on the fp32 kernels needs gigabytes of scratch: refused before any launch
    p = dk.make_params(1, 8, 131072, 64, 64, 512, 64, io_dtype=dk.DARK_BF16, path=dk.PATH_F32)
    assert dk.workspace_bytes(p, dk.OP_ATTN_FWD) > dk.static_scratch_bytes()
    import ctypes
    A = 1 << 20
    assert dk.lib().dark_attn_fwd_static(ctypes.byref(p), A, A, A, A, A, A, None) == dk.DARK_ESCRATCH
