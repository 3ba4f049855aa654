"""The column-sum entry point that allocates nothing (gpt_stage_op_colsum_noalloc) against
gpt_stage_op_colsum, through the C-ABI: same kernels and summation order, so the bits must
agree.  Two calls in a row, the second on a smaller input, so that stale contents of the
library's fixed scratch array would show."""
import numpy as np
import pytest
import torch

from paper_2507_19845_amd import binding as B
from paper_2507_19845_amd import synth

pytestmark = pytest.mark.gpu


def _both(dtype, M, N, tag):
    dt = B.GPTS_BF16 if dtype == "bf16" else B.GPTS_FP32
    A = B.to_device(synth.to_storage(synth.make_aux(0, tag, (M, N)), dtype), dtype)
    pre = synth.make_aux(0, tag + 1, (N,)).astype(np.float32)          # colsum accumulates (+=)
    want, got = torch.from_numpy(pre).cuda(), torch.from_numpy(pre).cuda()
    part = torch.empty(B.gpt_stage_op_colsum_scratch_bytes(M, N), dtype=torch.uint8, device="cuda")
    B.gpt_stage_op_colsum(dt, M, N, A, want, part)
    B.gpt_stage_op_colsum_noalloc(dt, M, N, A, got)
    torch.cuda.synchronize()
    return want.cpu().numpy(), got.cpu().numpy(), A


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_colsum_noalloc_matches_colsum_twice_in_a_row(dtype):
    print(f"[case] colsum_noalloc {dtype}", flush=True)
    for tag, (M, N) in enumerate([(4096, 16384), (300, 136)]):      # the second call is smaller
        want, got, A = _both(dtype, M, N, 40 + 2 * tag)
        assert np.array_equal(want, got), (dtype, M, N)
        ref = B.to_host(A).sum(0)
        # and both are the column sums (fp32 accumulation of M terms)
        assert np.abs(got - (synth.make_aux(0, 41 + 2 * tag, (N,)).astype(np.float64) + ref)).max() < 1e-3 * max(1.0, np.abs(ref).max())


def test_colsum_noalloc_rejects_sizes_beyond_its_array():
    A = torch.zeros((8, 16392), dtype=torch.float32, device="cuda")
    out = torch.zeros(16392, dtype=torch.float32, device="cuda")
    with pytest.raises(B.GptStageError) as ei:
        B.gpt_stage_op_colsum_noalloc(B.GPTS_FP32, 8, 16392, A, out)
    assert ei.value.code == B.GPTS_ESHAPE and "16384" in str(ei.value)
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0      # nothing was launched
