"""The entry point that allocates nothing: pserve_patch_mse_static against pserve_patch_mse.

Both run the same kernels in the same order, so the results agree bit for bit; the static form keeps its partial
sums in a fixed array of the library's device image.  Two calls in a row, the second on a smaller batch (the array
then still holds the first call's partial sums behind the part the second call uses)."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2501_09253_amd as ps
import workloads as wl
from oracle import cache as oc
from harness import to_dev

pytestmark = pytest.mark.gpu


def _images(seed, res, C_):
    return [wl.bf16_round(wl.Stream(seed, f"m{i}").normal((C_, h, w))) for i, (h, w) in enumerate(res)]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_patch_mse_static_two_calls(dtype):
    Cc = 64
    cases = [([(32, 32), (16, 48), (16, 16), (64, 32)], 8, 8), ([(16, 16), (8, 24)], 8, 8)]     # 68 patches, then 7
    for k, (res, ph, pw) in enumerate(cases):
        a, b = _images(10 + k, res, Cc), _images(20 + k, res, Cc)
        plan = ps.Plan(res, ph, pw)
        xa = plan.split([to_dev(t, dtype) for t in a])
        xb = plan.split([to_dev(t, dtype) for t in b])
        want = plan.patch_mse(xa, xb)
        out = torch.full((plan.P,), -1.0, dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_stats()["allocation.all.allocated"]           # allocations made so far (a count)
        got = plan.patch_mse_static(xa, xb, out=out)
        torch.cuda.synchronize()
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
        assert torch.equal(got, want), (k, dtype)
        ref = oc.patch_mse(a, b, ph, pw)
        assert np.abs(got.cpu().numpy().astype(np.float64) - ref).max() <= 2e-5 * np.abs(ref).max(), (k, dtype)
        plan.close()


def test_patch_mse_static_rejects_oversized_plan():
    res = [(4, 4 * (ps.binding.MSE_STATIC_MAX_PATCHES + 1))]
    plan = ps.Plan(res, 4, 4)
    assert plan.P == ps.binding.MSE_STATIC_MAX_PATCHES + 1
    x = torch.zeros((plan.T, 8), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ps.PserveError) as e:
        plan.patch_mse_static(x, x)
    assert e.value.status == -1 and "scratch" in str(e.value)
    plan.close()
