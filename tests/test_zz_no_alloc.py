"""The entry point that allocates nothing (dp_op_colsum_static: partial sums in a device array
inside the library) against dp_op_colsum, which takes a workspace: same kernels, so the same
bits; and against the plain column sums within one output rounding.  Two calls in a row, the
second on a smaller input (the array keeps the first call's partials)."""
import numpy as np
import pytest
import torch

import synthetic as syn
from paper_2505_05856_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = {torch.float32: 2e-5, torch.bfloat16: 8e-3}


def make(rows, cols, seed, dt):
    a = syn.normal(seed, 0, rows * cols).reshape(rows, cols).astype(np.float32)
    if dt == torch.bfloat16:
        a = syn.round_to_bf16(a)
    return a, torch.from_numpy(a).to(DEV).to(dt).contiguous()


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
def test_static_scratch_column_sums_match_the_workspace_form(dt):
    for rows, cols, seed in ((9000, 1032, 41), (700, 264, 42)):      # the second call is the smaller one
        a, t = make(rows, cols, seed, dt)
        want = torch.empty(cols, dtype=dt, device=DEV)
        ws = torch.empty(B.op_workspace_bytes(rows, cols), dtype=torch.uint8, device=DEV)
        B.op_colsum(t, want, ws)
        got = torch.full((cols,), float("nan"), dtype=dt, device=DEV)
        B.op_colsum_static(t, got)
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.int16 if dt == torch.bfloat16 else torch.int32),
                           want.view(torch.int16 if dt == torch.bfloat16 else torch.int32)), (rows, cols)
        ref = a.astype(np.float64).sum(axis=0)
        err = np.abs(got.float().cpu().numpy().astype(np.float64) - ref).max() / np.abs(ref).max()
        assert err < TOL[dt], (rows, cols, err)


def test_static_scratch_limits_and_empty_input():
    # no rows: zeros, nothing read
    out = torch.full((64,), float("nan"), dtype=torch.float32, device=DEV)
    B.op_colsum_static(torch.zeros(1, 64, dtype=torch.float32, device=DEV)[:0], out)
    torch.cuda.synchronize()
    assert torch.equal(out, torch.zeros_like(out))
    # beyond the array: refused with a message, nothing launched
    big = torch.zeros(16384, 8192, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(B.DpError) as e:
        B.op_colsum_static(big, torch.empty(8192, dtype=torch.bfloat16, device=DEV))
    assert e.value.status == "DP_E_UNSUPPORTED" and "static scratch" in str(e.value)
    # the largest width that fits at any row count
    t = torch.ones(16384, 4096, dtype=torch.bfloat16, device=DEV)
    out = torch.empty(4096, dtype=torch.bfloat16, device=DEV)
    B.op_colsum_static(t, out)
    torch.cuda.synchronize()
    assert torch.equal(out, torch.full_like(out, 16384.0))
