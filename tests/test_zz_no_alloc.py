"""The entry point that allocates nothing (static device scratch) against the
entry point it is a variant of (scratch in a caller workspace): two calls in a
row, the second smaller, each compared bit for bit and against the definition."""
import pytest
import torch

import workloads as WL
from tests.helpers import rel_err

pytestmark = pytest.mark.gpu


def _rand(seed, name, shape, std=1.0):
    return WL.seeded_normal_bf16(seed, name, shape, 0.0, std)


@pytest.mark.parametrize("out_f32", [True, False])
def test_static_scratch_gemm_matches_workspace_gemm(out_f32):
    from paper_2410_03960_amd import binding as B
    dt = torch.float32 if out_f32 else torch.bfloat16
    # first a call whose K is split over workgroups (few column tiles, many rows), then a smaller one
    # that takes other splits and leaves most of the first call's partial sums in the scratch
    for M, N, K in ((80, 1024, 4096), (49, 1056, 4096), (33, 192, 520), (64, 4096, 1376), (1, 16, 8)):
        A, W = _rand(41, f"A{M}x{K}", (M, K)).cuda(), _rand(42, f"W{N}x{K}", (N, K), 0.05).cuda()
        want = B.op_gemm_rows(A, W, out_f32=out_f32)
        out = torch.full((M, N), float("nan"), dtype=dt, device="cuda")
        got = B.op_gemm_rows_static(A, W, out)
        torch.cuda.synchronize()
        assert torch.equal(got, want), (M, N, K)
        ref = A.double().cpu() @ W.double().cpu().T
        assert rel_err(got.cpu(), ref) <= (1e-5 if out_f32 else 4e-3), (M, N, K)


def test_static_scratch_gemm_rejects_sizes_beyond_its_maximum():
    from paper_2410_03960_amd import binding as B
    W = _rand(2, "W", (8208, 64)).cuda()
    for M, Wt in ((81, W[:64]), (8, W)):          # too many rows; too many columns
        A = _rand(1, f"A{M}", (M, 64)).cuda()
        out = torch.empty((M, Wt.shape[0]), dtype=torch.float32, device="cuda")
        with pytest.raises(B.SwiftKVError) as e:
            B.op_gemm_rows_static(A, Wt.contiguous(), out)
        assert e.value.code == B.SWIFTKV_EINVAL and "static scratch" in str(e.value)
