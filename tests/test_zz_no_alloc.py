"""The allocation-free gate entry point (static device scratch) against the workspace entry point."""
import numpy as np
import pytest
import torch

from paper_2601_16515_amd import binding as sb
from paper_2601_16515_amd import workloads as wl

from .gpu_util import say

pytestmark = pytest.mark.gpu


def _case(B, N, D, seed):
    x = wl.round_to_bf16(wl.normal(seed, "x", (B, N, D)))
    w = wl.normal(seed, "w", (D,), std=0.05)
    return x, w, torch.from_numpy(x).cuda().to(torch.bfloat16), torch.from_numpy(w).cuda()


def test_static_scratch_gate_matches_workspace_gate(oracle):
    """Two calls in a row through the static buffer, the second on a smaller input (fewer partial sums than the
    first call left behind), each compared with salad_gate_fwd bit for bit and with the oracle to its bar."""
    for B, N, D, seed in ((3, 9000, 1536, 11), (2, 270, 512, 12)):
        say(f"static gate: B={B} N={N} D={D}")
        x_np, w_np, x, w = _case(B, N, D, seed)
        ref = sb.salad_gate_fwd(x, w, 0.125)
        s = torch.full((B,), float("nan"), dtype=torch.float32, device="cuda")
        sb.salad_gate_fwd_static(x, w, s, 0.125)
        torch.cuda.synchronize()
        assert np.array_equal(s.cpu().numpy(), ref.cpu().numpy())
        want = oracle.gate(x_np, w_np, 0.125)
        assert np.abs(s.cpu().numpy().astype(np.float64) - want).max() < 2e-6


def test_static_scratch_gate_rejects_what_does_not_fit():
    _, _, x, w = _case(1, 64, 64, 13)
    s = torch.empty(40, dtype=torch.float32, device="cuda")
    L = sb.lib()
    # B = 40: 40 * 512 partial sums do not fit the 64 KB buffer; refused on the host, nothing launched
    st = L.salad_gate_fwd_static(x.data_ptr(), w.data_ptr(), 0.0, 40, 32760, 64, sb.SALAD_BF16, s.data_ptr(), None)
    assert st == sb.SALAD_ENOSPC and "static" in L.salad_last_error().decode()
