"""GPU parity of pserve_split_stats: the split that also takes the statistics of the block's first normalisation.

The token matrix must be the one pserve_split writes, bit for bit, and the forward call that follows must meet the
oracle at the usual bar: whole-image statistics ("Patch-Tailored Diffusion Operators"), here merged from per-channel
moments of token chunks instead of a pass of their own.  Cases: patch shapes whose 32-token tiles divide into 8, 4, 2
and 1 chunks, widths of one and of several 64-channel slabs with groups that straddle the slabs (C = 320, G = 32),
inputs whose mean is far from zero, a reuse mask (the first norm of a residual block reads the fresh input on every
patch), a first stage that is an attention stage, and the shapes the fast path does not cover (fp32, narrow patches),
where the call must behave as the plain split.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import block as ob
from harness import GpuRun, rel_err, tolerance

pytestmark = pytest.mark.gpu


def _oracle(w, reuse=None, cache=None):
    cfg = w.cfg
    return ob.forward_batch(w.images, cfg.stages, w.params, G=cfg.G, heads=cfg.heads, eps=cfg.eps, ctx=w.ctx,
                            reuse=reuse, cache=cache, temb=w.temb)


def _forward_with_split_stats(run, reuse=None):
    x2 = torch.empty_like(run.x)
    run.plan.split(run.images, out=x2, cache=run.cache)
    assert torch.equal(x2.view(torch.int16) if x2.dtype == torch.bfloat16 else x2,
                       run.x.view(torch.int16) if run.x.dtype == torch.bfloat16 else run.x), "x differs from pserve_split"
    mask = run.plan_mask(reuse) if reuse is not None else None
    y = run.cache.forward(x2, run.ctx, mask, temb=run.temb)
    torch.cuda.synchronize()
    return y


CASES = [
    # (resolutions, patch, C, G, heads, stages)
    ([(32, 32), (16, 48), (16, 16)], (16, 16), 320, 32, 5, (wl.RES2,)),           # 8 tiles per patch: 8 chunks; groups straddle slabs
    ([(16, 32), (8, 8), (24, 16)], (8, 8), 64, 8, 1, (wl.RES2,)),                 # 2 tiles: 2 chunks, one slab
    ([(8, 24), (16, 8)], (4, 8), 128, 32, 2, (wl.RES1,)),                         # 1 tile: 1 chunk
    ([(32, 96), (64, 32)], (32, 32), 64, 4, 1, (wl.RES2,)),                       # 32 tiles: 8 chunks of 4 tiles
    ([(16, 48), (48, 24)], (16, 24), 128, 8, 2, (wl.RES1, wl.SATTN)),             # 12 tiles: 4 chunks of 3
    ([(16, 16), (32, 16), (16, 32)], (16, 16), 128, 16, 2, (wl.SATTN,)),          # first stage an attention stage
]


@pytest.mark.parametrize("case", range(len(CASES)))
def test_split_stats_matches_oracle(case):
    res, patch, C, G, heads, stages = CASES[case]
    cfg = wl.custom_config(res, patch, C=C, G=G, heads=heads, stages=stages, dtype="bf16", seed=70 + case)
    w = wl.make_workload(cfg)
    run = GpuRun(w)
    y_plain = run.forward()
    y = _forward_with_split_stats(run)
    got = [a.float().cpu().numpy() for a in run.plan.reassemble(y)]
    ref, _ = _oracle(w)
    err = rel_err(got, ref)
    # against the path with a statistics pass of its own: the same moments up to fp32 rounding order
    dev = float((y.float() - y_plain.float()).abs().max() / y_plain.float().abs().max())
    print(f"split_stats case {case}: rel err {err:.3e}, against the separate pass {dev:.3e}")
    assert err < tolerance("bf16")
    assert dev < 1e-2
    # single use: a second forward call on the same x takes its own statistics and must agree as well
    y3 = run.cache.forward(run.x, run.ctx, None, temb=run.temb)
    torch.cuda.synchronize()
    assert torch.equal(y3.view(torch.int16), y_plain.view(torch.int16))


@pytest.mark.parametrize("offset", [30.0, -30.0])
def test_split_stats_offset_input(offset):
    """Inputs with mean = 30 standard deviations: the chunk moments are taken around the chunk's first token."""
    cfg = wl.custom_config([(32, 32), (16, 48), (16, 16)], (16, 16), C=320, G=32, heads=5, stages=(wl.RES2,), dtype="bf16", seed=77)
    w = wl.make_workload(cfg)
    w.images = [wl.bf16_round(im + np.float32(offset)) for im in w.images]
    run = GpuRun(w)
    y = _forward_with_split_stats(run)
    got = [a.float().cpu().numpy() for a in run.plan.reassemble(y)]
    ref, _ = _oracle(w)
    err = rel_err(got, ref)
    print(f"split_stats offset {offset}: rel err {err:.3e}")
    assert err < tolerance("bf16")


def test_split_stats_with_reuse_mask():
    """With a mask the residual block's first norm still reads the fresh input on every patch, so the moments taken
    while splitting stay valid; reused patches keep the cached output bit for bit."""
    cfg = wl.custom_config([(32, 32), (16, 48), (16, 16)], (16, 16), C=128, G=8, heads=2, stages=(wl.RES2, wl.SATTN), dtype="bf16",
                           reuse_p=0.4, seed=78)
    w = wl.make_workload(cfg)
    run = GpuRun(w)
    run.load_cache()
    y = _forward_with_split_stats(run, reuse=w.reuse)
    got = [a.float().cpu().numpy() for a in run.plan.reassemble(y)]
    ref, _ = _oracle(w, reuse=w.reuse, cache=w.cache)
    assert rel_err(got, ref) < tolerance("bf16")
    for g, cy, m, (h, wd) in zip(got, w.cache["y"], w.reuse, cfg.resolutions):
        ph, pw = cfg.patch
        for r in range(h // ph):
            for c in range(wd // pw):
                if m[r, c]:
                    assert np.array_equal(g[:, r * ph:(r + 1) * ph, c * pw:(c + 1) * pw], cy[:, r * ph:(r + 1) * ph, c * pw:(c + 1) * pw])


@pytest.mark.parametrize("dtype,patch", [("f32", (8, 8)), ("bf16", (4, 4))])
def test_split_stats_falls_back(dtype, patch):
    """fp32, or patches whose width is no multiple of eight: the call is the plain split and the forward call takes its
    own statistics; the result is that of the ordinary path, bit for bit."""
    cfg = wl.custom_config([(16, 16), (8, 24)], patch, C=64, G=8, heads=1, stages=(wl.RES2,), dtype=dtype, seed=79)
    w = wl.make_workload(cfg)
    run = GpuRun(w)
    y_plain = run.forward()
    y = _forward_with_split_stats(run)
    assert torch.equal(y.view(torch.int32) if dtype == "f32" else y.view(torch.int16),
                       y_plain.view(torch.int32) if dtype == "f32" else y_plain.view(torch.int16))


def test_split_stats_config2_full():
    """Baseline configuration 2 at full size through the split that takes the statistics."""
    cfg = wl.config(2)
    w = wl.make_workload(cfg)
    run = GpuRun(w)
    y = _forward_with_split_stats(run)
    got = [a.float().cpu().numpy() for a in run.plan.reassemble(y)]
    ref, _ = _oracle(w)
    err = rel_err(got, ref)
    print(f"split_stats config 2: rel err {err:.3e}")
    assert err < tolerance("bf16")
