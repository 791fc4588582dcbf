"""GPU parity of the joint text-image block (PSERVE_MMDIT on a joint plan, through the C ABI) against oracle.block.mmdit
run on every request on its own.  Bars: fp32 1e-4, bf16 2e-2 of max|ref| (image and text outputs)."""
import numpy as np
import pytest
import torch

import paper_2501_09253_amd as ps
import workloads as wl
from oracle import block as ob
from harness import to_dev, to_host, tolerance

pytestmark = pytest.mark.gpu

NAMES = ("wm", "bm", "wq", "wk", "wv", "wo", "bo", "w1", "b1", "w2", "b2")


def make_params(seed, C, D, Fh, dtype, stage=0):
    rd = wl.bf16_round if dtype == "bf16" else (lambda a: a)
    g = lambda name, shape, scale: rd((wl.Stream(seed, f"{stage}.{name}").normal(shape) * scale).astype(np.float32))
    p = {}
    for X in ("img", "txt"):
        p[X + ".wm"], p[X + ".bm"] = g(X + "wm", (D, 6 * C), D ** -0.5), g(X + "bm", (6 * C,), 0.1)
        for n in ("wq", "wk", "wv", "wo"):
            p[X + "." + n] = g(X + n, (C, C), C ** -0.5)
        p[X + ".bo"] = g(X + "bo", (C,), 0.1)
        p[X + ".w1"], p[X + ".b1"] = g(X + "w1", (C, Fh), C ** -0.5), g(X + "b1", (Fh,), 0.1)
        p[X + ".w2"], p[X + ".b2"] = g(X + "w2", (Fh, C), Fh ** -0.5), g(X + "b2", (C,), 0.1)
    return p


def run_case(res, patch, C, heads, L, D, dtype, n_stages=1, mult=2, seed=81):
    rd = wl.bf16_round if dtype == "bf16" else (lambda a: a)
    imgs = [rd(wl.Stream(seed, f"i{k}").normal((C, h, w))) for k, (h, w) in enumerate(res)]
    text = rd(wl.Stream(seed, "txt").normal((len(res), L, C)))
    cvec = rd(wl.Stream(seed, "c").normal((len(res), D)))
    params = [make_params(seed, C, D, mult * C, dtype, s) for s in range(n_stages)]
    dt = ps.BF16 if dtype == "bf16" else ps.F32
    plan = ps.Plan(res, patch[0], patch[1], text_len=L)
    block = ps.Block(("MMDIT",) * n_stages, [{k: to_dev(v, dtype) for k, v in p.items()} for p in params], C_=C, G=1,
                     heads=heads, dtype=dt, ffn_mult=mult, temb_dim=D)
    cache = ps.Cache(plan, block, False)
    x = plan.split([to_dev(z, dtype) for z in imgs])
    x[np.repeat(plan.table("patch_rc")[:, 0] < 0, plan.ph * plan.pw)] = 0          # text patches: defined before the scatter
    plan.text_scatter(to_dev(text, dtype), x)
    y = cache.forward(x, None, None, temb=to_dev(cvec, dtype))
    torch.cuda.synchronize()
    got_i = [to_host(a) for a in plan.reassemble(y)]
    got_t = to_host(plan.text_gather(y))
    worst = 0.0
    for i, z in enumerate(imgs):
        ri, rt = z.astype(np.float64), text[i].astype(np.float64)
        for p in params:
            ri, rt = ob.mmdit(ri, rt, cvec[i], p, heads, 1e-5)
        scale = max(np.abs(ri).max(), np.abs(rt).max())
        worst = max(worst, np.abs(got_i[i] - ri).max() / scale, np.abs(got_t[i] - rt).max() / scale)
    assert np.isfinite(to_host(y)).all()                                           # padding rows stay finite
    return worst


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("res,patch,C,heads,L,D", [
    ([(8, 8), (4, 8), (8, 8)], (4, 4), 32, 2, 20, 12),             # two text patches, last one ragged
    ([(8, 8), (16, 8)], (8, 8), 64, 1, 7, 16),                     # text shorter than a patch, head dim 64
    ([(6, 10)], (6, 10), 24, 3, 60, 8),                            # text exactly one patch; odd widths
])
def test_joint_block_small(res, patch, C, heads, L, D, dtype):
    if dtype == "bf16" and C % 8:
        pytest.skip("bf16 rows must be multiples of 16 bytes")
    assert run_case(res, patch, C, heads, L, D, dtype) < tolerance(dtype)


def test_two_joint_blocks_in_a_row():
    assert run_case([(8, 8), (8, 16)], (4, 4), 32, 2, 10, 12, "f32", n_stages=2) < 1e-4


@pytest.mark.parametrize("res,patch,C,L", [([(32, 32), (16, 48), (16, 16)], (16, 16), 128, 77),
                                           ([(32, 32), (64, 32)], (16, 16), 256, 154)])
def test_joint_block_mfma_shapes_bf16(res, patch, C, L):
    assert run_case(res, patch, C, C // 64, L, 96, "bf16", mult=4) < 2e-2


def test_joint_block_needs_a_joint_plan():
    p = make_params(1, 32, 8, 64, "f32")
    block = ps.Block(("MMDIT",), [{k: to_dev(v, "f32") for k, v in p.items()}], C_=32, G=1, heads=2, dtype=ps.F32,
                     ffn_mult=2, temb_dim=8)
    with pytest.raises(ps.PserveError):
        ps.Cache(ps.Plan([(8, 8)], 4, 4), block, False)                            # plain plan
    with pytest.raises(ps.PserveError):
        ps.Cache(ps.Plan([(8, 8)], 4, 4, text_len=5), block, True)                 # no cache slots for joint blocks


def test_joint_block_config9_size():
    """Configuration 9 (C = 1536, 24 heads, 154 text tokens, four latents up to 64 x 64) through the shared harness."""
    from harness import GpuRun
    cfg = wl.config(9)
    w = wl.make_workload(cfg)
    run = GpuRun(w)
    y = run.forward()
    got_i = [to_host(a) for a in run.plan.reassemble(y)]
    got_t = to_host(run.plan.text_gather(y))
    worst = 0.0
    for i, z in enumerate(w.images):
        ri, rt = ob.mmdit(z, w.ctx[i], w.temb[i], w.params[0], cfg.heads, cfg.eps)
        scale = max(np.abs(ri).max(), np.abs(rt).max())
        worst = max(worst, np.abs(got_i[i] - ri).max() / scale, np.abs(got_t[i] - rt).max() / scale)
    print(f"config 9: rel err {worst:.3e}")
    assert worst < 2e-2
