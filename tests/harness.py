"""Test / bench harness: moves a seeded Workload to the GPU, runs the HIP path, brings results back.

Holds no arithmetic of the method: uploads, calls through the binding, downloads, compares.
"""
from __future__ import annotations

import numpy as np
import torch

import paper_2501_09253_amd as ps
import workloads as wl

SLOT_IDS = {"h1": ps.SLOT_H1, "r": ps.SLOT_R, "K": ps.SLOT_K, "V": ps.SLOT_V}


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16).contiguous() if dtype == "bf16" else t.contiguous()


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy()


class GpuRun:
    """One workload resident on the GPU with its plan, block and cache objects."""

    def __init__(self, w: wl.Workload, with_slots=None, patch=None):
        cfg = w.cfg
        self.w, self.cfg = w, cfg
        ph, pw = patch if patch is not None else cfg.patch
        self.joint = "MMDIT" in cfg.stages                     # text tokens ride along as extra patches
        self.plan = ps.Plan(cfg.resolutions, ph, pw, text_len=cfg.ctx_len if self.joint else 0)
        self.dtype = ps.BF16 if cfg.dtype == "bf16" else ps.F32
        self.images = [to_dev(im, cfg.dtype) for im in w.images]
        self.params = [{k: to_dev(v, cfg.dtype) for k, v in p.items()} for p in w.params]
        self.ctx = to_dev(w.ctx, cfg.dtype) if w.ctx is not None else None
        self.temb = to_dev(w.temb, cfg.dtype) if w.temb is not None else None
        self.block = ps.Block(cfg.stages, self.params, C_=cfg.C, G=cfg.G, heads=cfg.heads, dtype=self.dtype,
                              eps=cfg.eps, ctx_len=cfg.ctx_len, ctx_dim=cfg.ctx_dim, ffn_mult=cfg.ffn_mult,
                              temb_dim=cfg.temb_dim)
        if with_slots is None:
            with_slots = w.cache is not None
        self.cache = ps.Cache(self.plan, self.block, with_slots)
        self.x = self.plan.split(self.images)
        if self.joint:
            self.x[np.repeat(self.plan.table("patch_rc")[:, 0] < 0, self.plan.ph * self.plan.pw)] = 0
            self.plan.text_scatter(self.ctx, self.x)

    def plan_mask(self, reuse) -> torch.Tensor:
        """Per-request [gh, gw] bool grids (caller order) -> uint8 [P] in plan order."""
        owner, rc, perm = self.plan.table("patch_owner"), self.plan.table("patch_rc"), self.plan.table("perm")
        m = np.zeros(self.plan.P, dtype=np.uint8)
        for p in range(self.plan.P):
            m[p] = reuse[perm[owner[p]]][rc[p, 0], rc[p, 1]]
        return torch.from_numpy(m).cuda()

    def load_cache(self, cache=None):
        cache = cache if cache is not None else self.w.cache
        for name, per_image in cache.items():
            t = self.plan.split([to_dev(a, self.cfg.dtype) for a in per_image])
            if name == "y":
                self.cache.load(-1, ps.SLOT_Y, t)
            else:
                si, sl = name.split(".")
                self.cache.load(int(si), SLOT_IDS[sl], t)

    def read_cache(self):
        out = {}
        for name in self.w.cache:
            if name == "y":
                t = self.cache.read(-1, ps.SLOT_Y)
            else:
                si, sl = name.split(".")
                t = self.cache.read(int(si), SLOT_IDS[sl])
            out[name] = [to_host(a) for a in self.plan.reassemble(t)]
        return out

    def forward(self, reuse=None):
        mask = self.plan_mask(reuse) if reuse is not None else None
        y = self.cache.forward(self.x, None if self.joint else self.ctx, mask, temb=self.temb)
        torch.cuda.synchronize()
        return y

    def forward_images(self, reuse=None):
        y = self.forward(reuse)
        return [to_host(a) for a in self.plan.reassemble(y)]


def rel_err(got, ref) -> float:
    """max |got - ref| / max |ref| over a list of arrays."""
    num = max(float(np.abs(np.asarray(g, dtype=np.float64) - r).max()) for g, r in zip(got, ref))
    den = max(float(np.abs(r).max()) for r in ref)
    return num / den


def tolerance(dtype: str) -> float:
    return 2e-2 if dtype == "bf16" else 1e-4
