"""The hot path under HIP graph capture: split + pserve_block_forward + reassemble recorded once and replayed.

The forward call allocates nothing and clears nothing with memset, and its side stream (text key/value projection)
forks from and joins the captured stream through events, so a capture of the caller's stream holds the whole step.
Every replay is compared bit for bit with the eager result, with eager work between the replays."""
import numpy as np
import pytest
import torch

import paper_2501_09253_amd as ps
import workloads as wl
from harness import GpuRun, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("stages,reuse,stats", [((wl.RES2, wl.SATTN), False, False), ((wl.LSATTN, wl.LXATTN, wl.LFFN), False, False),
                                                ((wl.RES2, wl.SATTN), True, False), ((wl.RES2, wl.SATTN), False, True),
                                                ((wl.RES2, wl.SATTN), True, True)])
def test_step_replayed_from_a_graph_equals_eager(stages, reuse, stats):
    """stats: the split that also takes the first norm's moments (pserve_split_stats); the forward call recorded behind
    it merges them, in the capture as in the eager step."""
    cfg = wl.custom_config([(32, 32), (16, 48), (16, 16)], (16, 16), C=128, G=32, heads=2, stages=stages, dtype="bf16",
                           ctx_len=77, ctx_dim=128, reuse_p=0.4 if reuse else 0.0, seed=71)
    w = wl.make_workload(cfg)
    run = GpuRun(w)
    mask = None
    if reuse:
        run.load_cache()
        mask = run.plan_mask(w.reuse)
    ps.profile_enable(False)
    x = torch.empty((run.plan.T, cfg.C), dtype=torch.bfloat16, device="cuda")
    y = torch.empty_like(x)
    outs = [torch.empty_like(im) for im in run.images]

    def step():
        run.plan.split(run.images, out=x, cache=run.cache if stats else None)
        run.cache.forward(x, run.ctx, mask, y=y)
        run.plan.reassemble(y, images=outs)

    step()                                              # eager reference (also fills every slot once)
    torch.cuda.synchronize()
    ref = [o.clone() for o in outs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()                                          # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for k in range(4):
        for o in outs:
            o.zero_()
        y.zero_()
        g.replay()
        torch.cuda.synchronize()
        for o, r in zip(outs, ref):
            assert torch.equal(o, r), f"replay {k}"
        step()                                          # eager work between the replays
        torch.cuda.synchronize()
        for o, r in zip(outs, ref):
            assert torch.equal(o, r), f"eager after replay {k}"


def test_joint_block_replayed_from_a_graph_equals_eager():
    """A joint text-image block: its text stream's kernels run on the library's side stream, forked from and joined to
    the captured stream twice per stage; the capture must hold both streams' work."""
    cfg = wl.custom_config([(32, 32), (16, 48), (16, 16)], (16, 16), C=128, G=32, heads=2, stages=(wl.MMDIT, wl.MMDIT),
                           dtype="bf16", ctx_len=40, ctx_dim=128, seed=72, temb_dim=96)
    w = wl.make_workload(cfg)
    run = GpuRun(w)
    ps.profile_enable(False)
    x = run.x                                           # image rows from the split, text rows scattered in
    y = torch.empty_like(x)
    outs = [torch.empty_like(im) for im in run.images]

    def step():
        run.cache.forward(x, None, None, y=y, temb=run.temb)
        run.plan.reassemble(y, images=outs)

    step()
    torch.cuda.synchronize()
    ref = [o.clone() for o in outs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for k in range(4):
        for o in outs:
            o.zero_()
        y.zero_()
        g.replay()
        torch.cuda.synchronize()
        for o, r in zip(outs, ref):
            assert torch.equal(o, r), f"replay {k}"
        step()
        torch.cuda.synchronize()
        for o, r in zip(outs, ref):
            assert torch.equal(o, r), f"eager after replay {k}"
