"""GPU parity of the resolution changes between levels (through the C ABI) against oracle/resample.py: every image
on its own, unpatched.  Bars: fp32 1e-4, bf16 2e-2 of max|ref|."""
import numpy as np
import pytest
import torch

import paper_2501_09253_amd as ps
import workloads as wl
from oracle import resample as orr
from harness import to_dev, to_host, rel_err, tolerance

pytestmark = pytest.mark.gpu

CASES = [
    # resolutions, patch, C_in, C_out
    ([(8, 8), (16, 8), (8, 24)], (8, 8), 8, 16),              # one-patch images and patch rows / columns
    ([(12, 20), (4, 4)], (4, 4), 16, 8),                      # small patches: tiles span several patches and requests
    ([(32, 32), (16, 48)], (16, 16), 64, 128),                # MFMA shapes (bf16), wider output
    ([(32, 64)], (32, 32), 128, 64),                          # whole 32-wide rows, narrower output
    ([(6, 10), (6, 10)], (6, 10), 24, 40),                    # odd widths: reference kernels
]


def _params(seed, C_in, C_out, dtype):
    rd = wl.bf16_round if dtype == "bf16" else (lambda a: a)
    w = rd((wl.Stream(seed, "w").normal((C_out, C_in, 3, 3)) / np.sqrt(9.0 * C_in)).astype(np.float32))
    b = rd((0.1 * wl.Stream(seed, "b").normal((C_out,))).astype(np.float32))
    return w, b


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("kind", ["down2", "up2"])
@pytest.mark.parametrize("res,patch,C_in,C_out", CASES)
def test_resample_matches_per_image_operator(res, patch, C_in, C_out, kind, dtype):
    if dtype == "bf16" and (C_in % 8 or C_out % 8):
        pytest.skip("bf16 rows must be multiples of 16 bytes")
    rd = wl.bf16_round if dtype == "bf16" else (lambda a: a)
    imgs = [rd(wl.Stream(51, f"i{k}").normal((C_in, h, w))) for k, (h, w) in enumerate(res)]
    w, b = _params(52, C_in, C_out, dtype)
    ph, pw = patch
    plan_in = ps.Plan(res, ph, pw)
    if kind == "down2":
        plan_out = ps.Plan([(h // 2, w_ // 2) for h, w_ in res], ph // 2, pw // 2)
        ref = [orr.down2(z, w, b) for z in imgs]
        op = ps.Resample(ps.DOWN2, to_dev(w, dtype), to_dev(b, dtype), ps.BF16 if dtype == "bf16" else ps.F32)
    else:
        plan_out = ps.Plan([(2 * h, 2 * w_) for h, w_ in res], 2 * ph, 2 * pw)
        ref = [orr.up2(z, w, b) for z in imgs]
        op = ps.Resample(ps.UP2, to_dev(w, dtype), to_dev(b, dtype), ps.BF16 if dtype == "bf16" else ps.F32)
    x = plan_in.split([to_dev(z, dtype) for z in imgs])
    y = op.forward(plan_in, plan_out, x)
    torch.cuda.synchronize()
    got = [to_host(a) for a in plan_out.reassemble(y)]
    for g, r in zip(got, ref):
        assert g.shape == r.shape
    assert rel_err(got, ref) < tolerance(dtype)


def test_resample_rejects_mismatched_plans_and_small_workspace():
    w, b = _params(53, 8, 8, "f32")
    op = ps.Resample(ps.DOWN2, to_dev(w, "f32"), to_dev(b, "f32"), ps.F32)
    plan_in = ps.Plan([(8, 8), (16, 8)], 8, 8)
    x = torch.zeros((plan_in.T, 8), device="cuda")
    with pytest.raises(ps.PserveError):
        op.forward(plan_in, ps.Plan([(4, 4), (8, 8)], 4, 4), x)            # second request is not the halved one
    with pytest.raises(ps.PserveError):
        op.forward(plan_in, ps.Plan([(4, 4), (8, 4)], 2, 2), x)            # patch not halved
    good = ps.Plan([(4, 4), (8, 4)], 4, 4)
    with pytest.raises(ps.PserveError):
        op.forward(plan_in, good, x, workspace=torch.empty(64, dtype=torch.uint8, device="cuda"))
    odd = ps.Plan([(6, 10)], 3, 5)
    with pytest.raises(ps.PserveError):
        op.forward(odd, ps.Plan([(3, 5)], 3, 5), torch.zeros((odd.T, 8), device="cuda"))   # odd patch: cannot be halved


def test_down_then_up_at_config2_size():
    """Config 2's latents (C = 320) down to half size and back up, against the oracle chain."""
    cfg = wl.config(2)
    imgs = [wl.bf16_round(wl.Stream(61, f"i{k}").normal((cfg.C, h, w))) for k, (h, w) in enumerate(cfg.resolutions)]
    wd, bd = _params(62, cfg.C, cfg.C, "bf16")
    wu, bu = _params(63, cfg.C, cfg.C, "bf16")
    ph, pw = cfg.patch
    p_hi = ps.Plan(cfg.resolutions, ph, pw)
    p_lo = ps.Plan([(h // 2, w // 2) for h, w in cfg.resolutions], ph // 2, pw // 2)
    down = ps.Resample(ps.DOWN2, to_dev(wd, "bf16"), to_dev(bd, "bf16"), ps.BF16)
    up = ps.Resample(ps.UP2, to_dev(wu, "bf16"), to_dev(bu, "bf16"), ps.BF16)
    x = p_hi.split([to_dev(z, "bf16") for z in imgs])
    lo = down.forward(p_hi, p_lo, x)
    hi = up.forward(p_lo, p_hi, lo)
    torch.cuda.synchronize()
    ref_lo = [orr.down2(z, wd, bd) for z in imgs]
    assert rel_err([to_host(a) for a in p_lo.reassemble(lo)], ref_lo) < 2e-2
    # the second operator is checked on the GPU's own (bf16-rounded) intermediate
    lo_imgs = [to_host(a) for a in p_lo.reassemble(lo)]
    ref_hi = [orr.up2(z, wu, bu) for z in lo_imgs]
    assert rel_err([to_host(a) for a in p_hi.reassemble(hi)], ref_hi) < 2e-2
