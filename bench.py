"""Benchmark of the hot path: patch-tokens/s of one mixed-resolution denoising block on one MI355X.

A step = one pass of the whole hot path over one resident batch: split (per-image NCHW -> patch
batch), pserve_block_forward, reassembly (patch batch -> per-image NCHW), on a plan built once
for the batch composition (planner time is reported separately).  Inputs are resident in HBM
before the timed region.  One JSON line is printed.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 5] [--only]

The headline is configuration 5 (the largest single-GPU workload: the skewed batch with the patch cache); the line
also carries a short measurement of every baseline configuration 1..5 under "configs" (left out with --only, which
profiler runs use so that a trace holds one workload).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
EVENT_EVERY = 4                # the timed region brackets the dominant kernel in every 4th step

# HBM bytes per launch of the dominant kernel.  NOT measured by this run: counters need a profiler run of their own.
# The figures come from two rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE) of `python3 bench.py --config N --only`,
# each scaled by what the same counter reads for the 256 MiB calibration copy below; they are read from the committed
# summary of those runs, which is named beside the number in the output.  Kernel label -> kernel name in the summary.
PROFILE_KERNEL = {"conv3x3": "conv_mfma_kernel", "attn_self": "attn_pipe_kernel", "attn_cross": "attn_cross_kernel",
                  "ffn_geglu": "gemm_mfma_kernel<128, 128, true", "gn_stats": "gn_partial_kernel"}


def profiled_traffic(cfg_id, label):
    """(HBM bytes per launch, summary file) of kernel `label` from the committed counter summary of configuration
    cfg_id (the table "HBM traffic per launch": scaled read MB + scaled write MB of the first row whose kernel name
    matches), or (None, None) when there is no summary or no such row."""
    rel = f"profiles/bench_config{cfg_id}_kernels_traffic_counters.md"
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), rel)
    name = PROFILE_KERNEL.get(label)
    if name is None or not os.path.exists(path):
        return None, None
    in_table = False
    for line in open(path):
        if line.startswith("## "):
            in_table = line.startswith("## HBM traffic per launch")
        elif in_table and line.startswith("| pserve::" + name):
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            try:
                return (float(cells[-2]) + float(cells[-1])) * 1e6, rel
            except ValueError:
                return None, None
    return None, None


def kernel_work(cfg, n_active_tokens, patch=None):
    """Algorithmic work per LAUNCH of each kernel label: (flops, bytes).

    Units: tokens T (all patches) or computed tokens Ta; b = bytes per element; C channels.
      conv3x3      2*9*C*C flops per computed token; bytes 2*b*C per token (read a, write o) + 18*C*C weights
      linear_*     2*Cin*Cout flops per token
      attn_self    4*N_i*C flops per query token of image i
      attn_cross   4*L*C flops per token
      gn_stats     b*C bytes per token (one read); gn_finalize = the merge of partial moments alone (where the split pass or
                   the previous convolution left them behind): no tensor traffic
      gn_apply     2*b*C bytes per computed token (read + write); gn_apply_stitch: computed tokens plus the border tokens of
                   reused patches, and b*C*ring per patch (rim writes)
      halo_gather  2*b*C*ring bytes per patch (read + write of the ring)
      reuse_copy   2*b*C bytes per token
      layer_norm   2*b*C bytes per computed token (read + write)
    """
    b = 2 if cfg.dtype == "bf16" else 4
    C, T, Ta = cfg.C, cfg.T, n_active_tokens
    ph, pw = patch if patch is not None else cfg.patch
    ring = 2 * (pw + 2) + 2 * ph
    border = 2 * pw + 2 * (ph - 2) if ph > 1 else pw        # border tokens of a patch
    Pa = Ta // (ph * pw)
    P = T // (ph * pw)
    frac = Ta / T
    F = cfg.ffn_mult * C
    attn = sum(4.0 * (h * w) * (h * w) * C for h, w in cfg.resolutions) * frac
    if "MMDIT" in cfg.stages:
        # joint block: every linear kernel runs once per stream (image rows, text rows), one attention over both; the
        # per-launch figures below are the mean of the two launches
        L = cfg.ctx_len
        attn = sum(4.0 * (h * w + L) * (h * w + L) * C for h, w in cfg.resolutions)
        Ta = (T + cfg.n * L) / 2.0
    return {
        "conv3x3": (2.0 * 9 * C * C * Ta, 2.0 * b * C * Ta + 9.0 * b * C * C),
        "linear_qkv": (2.0 * C * 3 * C * Ta, b * 4.0 * C * Ta),
        "linear_out": (2.0 * C * C * Ta, b * 3.0 * C * Ta),
        "linear_q": (2.0 * C * C * Ta, b * 2.0 * C * Ta),
        "linear_ctx_kv": (2.0 * cfg.ctx_dim * 2 * C * cfg.n * cfg.ctx_len, 0.0),
        "ffn_geglu": (2.0 * C * 2 * F * Ta, b * (C + F) * Ta),
        "ffn_out": (2.0 * F * C * Ta, b * (F + 2 * C) * Ta),
        "attn_self": (attn, b * 4.0 * C * Ta),
        "attn_cross": (4.0 * cfg.ctx_len * C * Ta, b * 2.0 * C * Ta),
        "gn_stats": (0.0, 1.0 * b * C * T),
        "gn_apply": (0.0, 2.0 * b * C * Ta),
        "gn_apply_stitch": (0.0, 2.0 * b * C * (Ta + (P - Pa) * border) + 1.0 * b * C * ring * P),
        "halo_gather": (0.0, 2.0 * b * C * ring * Pa),
        "reuse_copy": (0.0, 2.0 * b * C * T),
        "layer_norm": (0.0, 2.0 * b * C * Ta),
        "mlp_in": (2.0 * C * F * Ta, b * (C + F) * Ta),
        "mlp_out": (2.0 * F * C * Ta, b * (F + 2 * C) * Ta),
    }


def big_workload(n_images):
    """The stage list and mask rate of configuration 5 on n_images latents of 256 x 256 (84 MB each at C = 640, bf16):
    tensors far beyond the 256 MB last-level cache, for the HBM-bound kernels.  Values from numpy's generator (the
    seeded counter streams of workloads.py take minutes at this size; the kernels' time does not depend on the values)."""
    import numpy as np
    import workloads as wl
    cfg = wl.custom_config([(256, 256)] * n_images, (32, 32), C=640, G=32, heads=10, stages=(wl.RES2, wl.SATTN),
                           dtype="bf16", reuse_p=0.4, seed=55)
    cfg.cfg_id, cfg.name = 0, f"hbm-sweep-{n_images}x256x256"
    rng = np.random.default_rng(55)
    draw = lambda shape: wl.bf16_round(rng.standard_normal(shape, dtype=np.float32))
    images = [draw((cfg.C, 256, 256)) for _ in range(n_images)]
    params = []
    for st in cfg.stages:
        d = {}
        for name, (shape, kind) in wl.stage_param_shapes(st, cfg).items():
            z = rng.standard_normal(shape, dtype=np.float32)
            if kind == "gamma":
                z = 1.0 + 0.1 * z
            elif kind in ("beta", "bias"):
                z = 0.1 * z
            else:
                z = z / np.float32(np.sqrt(float(kind.split(":")[1])))
            d[name] = wl.bf16_round(z.astype(np.float32))
        params.append(d)
    reuse = [rng.random((8, 8)) < cfg.reuse_p for _ in range(n_images)]
    names = [f"{si}.{sl}" for si, st in enumerate(cfg.stages) for sl in wl.stage_cache_slots(st)] + ["y"]
    one = draw((cfg.C, 256, 256))                      # every slot of every image: the same values (they are only copied)
    cache = {nm: [one for _ in range(n_images)] for nm in names}
    return wl.Workload(cfg, images, params, None, reuse, cache)


def measure(cfg_id, steps, warmup, all_kernels=False, events=True, patch=None, peaks=None, workload=None):
    """One configuration on the GPU: `warmup` untimed steps, then exactly `steps` timed ones.  Returns the result
    fields and the workload (for the CPU-baseline leg)."""
    import torch
    import paper_2501_09253_amd as ps
    import workloads as wl
    from harness import GpuRun

    if workload is not None:
        w, cfg = workload, workload.cfg
    else:
        cfg = wl.config(cfg_id)
        w = wl.make_workload(cfg)
    assert patch is None or w.reuse is None, "--patch cannot be combined with a reuse mask"
    run = GpuRun(w, patch=tuple(patch) if patch else None)
    patch = (run.plan.ph, run.plan.pw)
    torch.cuda.synchronize()
    mask = None
    n_active = cfg.T
    if w.reuse is not None:
        run.load_cache()
        mask = run.plan_mask(w.reuse)
        n_active = int((mask == 0).sum().item()) * patch[0] * patch[1]
    # planner time (one-off per batch composition)
    tp = time.perf_counter()
    for _ in range(5):
        p = ps.Plan(cfg.resolutions, *patch)
        p.close()
    plan_us = (time.perf_counter() - tp) / 5 * 1e6

    y = torch.empty_like(run.x)
    outs = [torch.empty_like(im) for im in run.images]

    def step():
        run.plan.split(run.images, out=run.x, cache=run.cache)      # also takes the first norm's statistics where it can
        run.cache.forward(run.x, None if run.joint else run.ctx, mask, y=y, temb=run.temb)
        run.plan.reassemble(y, outs)

    # Warm-up; its last steps are timed kernel by kernel to find the dominant kernel.  In the timed region only THAT
    # kernel is bracketed with HIP events (on the stream the library launches on): every event pair costs a few
    # microseconds of stream time, and bracketing all kernels would lower the very throughput being measured.
    for _ in range(max(0, warmup - 3)):
        step()
    torch.cuda.synchronize()
    dom = None
    prof_all = {}
    if events:
        ps.profile_select(None)
        ps.profile_enable(True)
    n_probe = min(3, warmup)
    for _ in range(n_probe):
        step()
    torch.cuda.synchronize()
    if events:
        prof_all = ps.profile_read() if n_probe else {}
        if all_kernels:                      # a longer untimed pass for the per-kernel table
            for _ in range(steps):
                step()
            torch.cuda.synchronize()
            more = ps.profile_read()
            prof_all = {k: {"calls": more[k]["calls"], "total_ms": more[k]["total_ms"]} for k in more}
            n_probe = steps
        if prof_all:
            dom = max(prof_all, key=lambda k: prof_all[k]["total_ms"])
        ps.profile_select(dom)
        ps.profile_sample(EVENT_EVERY)            # the dominant kernel of every 4th step: 2-3 us of event cost per step
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t1
    prof = ps.profile_read() if events else {}
    ps.profile_enable(False)
    ps.profile_select(None)
    ps.profile_sample(1)
    ms_per_step = dt / steps * 1e3

    # block-only time on the same stream, for reference
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        run.cache.forward(run.x, None if run.joint else run.ctx, mask, y=y, temb=run.temb)
    e1.record()
    torch.cuda.synchronize()
    block_ms = e0.elapsed_time(e1) / steps

    # cache-manager pieces (outside the step): the predictor's per-patch MSE feature, and with slots the migration of
    # every slot to a cache of the same batch (all requests common)
    extras = {}
    if all_kernels:
        def timed(fn, reps=20):
            fn()
            a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a0.record()
            for _ in range(reps):
                fn()
            a1.record()
            torch.cuda.synchronize()
            return a0.elapsed_time(a1) / reps * 1e3
        es = 2 if cfg.dtype == "bf16" else 4
        us = timed(lambda: run.plan.patch_mse(run.x, y))
        gbs = 2.0 * cfg.T * cfg.C * es / (us * 1e-6) / 1e9
        extras["patch_mse"] = {"avg_us": us, "gbs": gbs, "frac_hbm": gbs / PEAK_HBM_GBS}
        for name, fn in (("split", lambda: run.plan.split(run.images, out=run.x)),
                         ("split_stats", lambda: run.plan.split(run.images, out=run.x, cache=run.cache)),
                         ("reassemble", lambda: run.plan.reassemble(y, outs))):
            us = timed(fn)
            gbs = 2.0 * cfg.T * cfg.C * es / (us * 1e-6) / 1e9
            extras[name] = {"avg_us": us, "gbs": gbs, "frac_hbm": gbs / PEAK_HBM_GBS}
        if cfg.dtype == "bf16" and patch[0] % 2 == 0 and patch[1] % 2 == 0 and w.reuse is None and not run.joint:
            # the level changes at this configuration's size: C -> C, down to half size and back up (random weights)
            from harness import to_dev
            import numpy as _np
            wt = to_dev((wl.Stream(cfg.seed, "rs.w").normal((cfg.C, cfg.C, 3, 3)) / _np.sqrt(9.0 * cfg.C)).astype(_np.float32), "bf16")
            bt = to_dev(_np.zeros(cfg.C, dtype=_np.float32), "bf16")
            lo_plan = ps.Plan([(h // 2, w_ // 2) for h, w_ in cfg.resolutions], patch[0] // 2, patch[1] // 2)
            down, up = ps.Resample(ps.DOWN2, wt, bt, ps.BF16), ps.Resample(ps.UP2, wt, bt, ps.BF16)
            lo = down.forward(run.plan, lo_plan, run.x)
            us = timed(lambda: down.forward(run.plan, lo_plan, run.x, y=lo))
            tf = 2.0 * 9 * cfg.C * cfg.C * lo_plan.T / (us * 1e-6) / 1e12
            extras["down2"] = {"avg_us": us, "tflops": tf, "frac_mfma": tf / PEAK_BF16_TFLOPS}
            us = timed(lambda: up.forward(lo_plan, run.plan, lo, y=y))
            tf = 2.0 * 16 * cfg.C * cfg.C * lo_plan.T / (us * 1e-6) / 1e12      # four merged taps per output pixel
            extras["up2"] = {"avg_us": us, "tflops": tf, "frac_mfma": tf / PEAK_BF16_TFLOPS}
        if w.reuse is not None:
            ids = list(range(cfg.n))
            _, _, src = run.plan.cache_sets(ids, run.plan, ids)
            twin = ps.Cache(run.plan, run.block, True)
            us = timed(lambda: twin.migrate_from(run.cache, src), reps=5)
            n_slots = 1 + sum({"RES2": 1, "SATTN": 3}.get(s, 0) for s in cfg.stages)
            gbs = 2.0 * n_slots * cfg.T * cfg.C * es / (us * 1e-6) / 1e9
            extras["cache_migrate"] = {"avg_us": us, "slots": n_slots, "gbs": gbs, "frac_hbm": gbs / PEAK_HBM_GBS}
            twin.close()

    work = kernel_work(cfg, n_active, patch)

    def entry(name, rec, steps_):
        avg_ms = rec["total_ms"] / rec["calls"]
        fl, by = work.get(name, (0.0, 0.0))
        ent = {"calls_per_step": rec["calls"] / max(1, steps_), "avg_us": avg_ms * 1e3}
        if fl > 0:
            ent["tflops"] = fl / (avg_ms * 1e-3) / 1e12
            ent["frac_mfma"] = ent["tflops"] / PEAK_BF16_TFLOPS
        elif by > 0:
            ent["gbs"] = by / (avg_ms * 1e-3) / 1e9
            ent["frac_hbm"] = ent["gbs"] / PEAK_HBM_GBS
        return ent
    kernels = {name: entry(name, rec, n_probe) for name, rec in prof_all.items()}      # untimed pass (all kernels)
    timed_k = {name: entry(name, rec, max(1, (steps + EVENT_EVERY - 1) // EVENT_EVERY))    # timed region (dominant kernel)
               for name, rec in prof.items()}
    roofline = None
    if timed_k:
        if dom not in timed_k:                     # no warm-up steps: every kernel was timed in the timed region
            dom = max(prof, key=lambda k: prof[k]["total_ms"])
        ent = timed_k[dom]
        traffic, source = profiled_traffic(cfg.cfg_id, dom)
        mfma = "tflops" in ent
        measured_peak = None if peaks is None else peaks["mfma_bf16_tflops" if mfma else "copy_gbs"]
        achieved = ent["tflops"] if mfma else ent.get("gbs")
        roofline = {"kernel": dom, "bound": "mfma" if mfma else "hbm", "achieved": achieved,
                    "peak": PEAK_BF16_TFLOPS if mfma else PEAK_HBM_GBS, "unit": "TFLOP/s" if mfma else "GB/s",
                    "frac": ent["frac_mfma"] if mfma else ent.get("frac_hbm"),
                    "traffic": traffic, "traffic_source": source, "avg_us": ent["avg_us"],
                    "peak_measured": measured_peak,
                    "frac_of_measured": (achieved / measured_peak) if (measured_peak and achieved) else None}
        # the rate of a synthetic stream with this kernel's instruction mix (no memory, no barriers), where probed
        mix_peak = None if peaks is None else peaks.get({"attn_self": "attention_mix_tflops", "conv3x3": "conv_mix_tflops"}.get(dom))
        if mix_peak and achieved:
            roofline["peak_same_mix"] = mix_peak
            roofline["frac_of_same_mix"] = achieved / mix_peak
    res = {
        "ms_per_step": ms_per_step, "tokens_per_s": cfg.T / (ms_per_step * 1e-3),
        "workload": f"config{cfg.cfg_id} {cfg.name}: latents {sorted(set(cfg.resolutions))} x{cfg.n}, "
                    f"patch {patch[0]}x{patch[1]}, P={run.plan.P}, T={cfg.T}, C={cfg.C}, stages={'+'.join(cfg.stages)}"
                    + (f", reuse p={cfg.reuse_p} ({cfg.T - n_active} tokens reused)" if w.reuse is not None else ""),
        "block_ms": block_ms, "plan_us": plan_us, "n_active": n_active, "roofline": roofline, "kernels": kernels,
        "extras": extras, "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "T": cfg.T,
    }
    run.cache.close()
    run.block.close()
    run.plan.close()
    del run, y, outs
    torch.cuda.empty_cache()
    return res, w


def cpu_baseline(w):
    """The oracle as it stands on the host cores, on a bounded sample of the workload (about 10-25 s)."""
    from oracle import block as ob
    from threadpoolctl import threadpool_info
    cfg = w.cfg
    # bounded sample: whole images of the workload, smallest first, until ~20 s of oracle time
    order = sorted(range(cfg.n), key=lambda i: cfg.resolutions[i][0] * cfg.resolutions[i][1])
    done_tok, tc = 0, time.perf_counter()
    used = []
    passes = 0
    while time.perf_counter() - tc < 10.0:          # repeat whole passes until about 10 s of oracle time
        passes += 1
        for i in order:
            H, W = cfg.resolutions[i]
            if H * W > 16384 and used:
                continue                      # a 65,536-token image alone is minutes of fp64 attention
            c_i = None if w.cache is None else {k: v[i] for k, v in w.cache.items()}
            if "MMDIT" in cfg.stages:
                ob.mmdit(w.images[i], w.ctx[i], w.temb[i], w.params[0], cfg.heads, cfg.eps)
            else:
                ob.block_forward(w.images[i], cfg.stages, w.params, G=cfg.G, heads=cfg.heads, eps=cfg.eps,
                                 ctx=None if w.ctx is None else w.ctx[i],
                                 reuse=None if w.reuse is None else w.reuse[i], cache=c_i,
                                 temb=None if w.temb is None else w.temb[i])
            done_tok += H * W
            used.append(i)
            if time.perf_counter() - tc > 25.0:
                break
    cpu_s = time.perf_counter() - tc
    threads = max([t.get("num_threads", 1) for t in threadpool_info()] + [1])
    return {"value": done_tok / cpu_s, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"{passes} pass(es) over {len(set(used))} of {cfg.n} images ({done_tok} tokens in total), whole block, "
                      f"fp64 numpy, {cpu_s:.1f} s"}


def library_gemm(steps, warmup):
    """torch.matmul (the vendor library's tuned bf16 GEMM) on the shapes the block's MFMA kernels work on, with
    standard-normal operands: what a plain GEMM of that shape reaches on this chip, without any of the fused work
    (patch gather and halo of the convolution, bias / residual / GEGLU / transposed outputs of the linear layers).
    M of the convolutions: computed tokens; K: nine taps x C."""
    import torch
    shapes = [("config 2 conv3x3", 29696, 2880, 320),
              ("config 3 q/k/v", 13312, 640, 1920), ("config 3 attn out", 13312, 640, 640),
              ("config 3 ffn in (GEGLU)", 13312, 640, 5120), ("config 3 ffn out", 13312, 2560, 640),
              ("config 4 conv3x3", 13440, 11520, 1280), ("config 4 q/k/v", 13440, 1280, 3840), ("config 4 attn out", 13440, 1280, 1280),
              ("config 5 conv3x3", 78848, 5760, 640), ("config 5 q/k/v", 131072, 640, 1920), ("config 5 attn out", 78848, 640, 640)]
    gen = torch.Generator(device="cuda").manual_seed(5)
    rows = []
    for name, M, K, N in shapes:
        a = torch.randn(M, K, device="cuda", dtype=torch.bfloat16, generator=gen)
        b = torch.randn(N, K, device="cuda", dtype=torch.bfloat16, generator=gen)
        for _ in range(max(1, warmup)):
            c = a @ b.t()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(steps):
            c = a @ b.t()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / steps * 1e3
        rows.append({"shape": name, "M": M, "K": K, "N": N, "avg_us": us, "tflops": 2.0 * M * K * N / us / 1e6,
                     "frac": 2.0 * M * K * N / us / 1e6 / PEAK_BF16_TFLOPS})
        del a, b, c
    return rows


def library_attention(steps, warmup):
    """torch's fused attention (the vendor's flash-attention kernels) at head dimension 64, ten heads, on sequence
    lengths of the configurations' images (all queries computed, no reuse mask): 256 tokens (16 x 16 latents of
    configuration 3), 4,096 and 65,536 (the 64 x 64 and 256 x 256 latents of configuration 5)."""
    import torch
    import torch.nn.functional as F
    gen = torch.Generator(device="cuda").manual_seed(6)
    rows = []
    for name, B, S in (("64 x 256 tokens", 64, 256), ("16 x 4,096 tokens", 16, 4096), ("4 x 16,384 tokens", 4, 16384),
                       ("1 x 65,536 tokens", 1, 65536)):
        q, k, v = (torch.randn(B, 10, S, 64, device="cuda", dtype=torch.bfloat16, generator=gen) for _ in range(3))
        for _ in range(warmup):
            o = F.scaled_dot_product_attention(q, k, v)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(steps):
            o = F.scaled_dot_product_attention(q, k, v)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / steps * 1e3
        fl = 4.0 * B * 10 * S * S * 64
        rows.append({"shape": name, "heads": 10, "d": 64, "avg_us": us, "tflops": fl / us / 1e6, "frac": fl / us / 1e6 / PEAK_BF16_TFLOPS})
        del q, k, v, o
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=5, help="benchmark configuration 1..5 (default 5: the largest one, the skewed batch with cache reuse), 6 = config 3 with per-token LayerNorms, 7 = config 2 with the time embedding, 8 = a diffusion-transformer block, 9 = a joint text-image block")
    ap.add_argument("--patch", type=int, nargs=2, default=None, metavar=("PH", "PW"),
                    help="patch size override for the patch-size sweep (not for reuse configs: the mask is per patch)")
    ap.add_argument("--only", action="store_true", help="measure --config alone: no \"configs\" array, no peak probes (profiler runs)")
    ap.add_argument("--hbm-sweep", type=int, nargs="+", default=None, metavar="N",
                    help="instead of a configuration: the HBM-bound kernels on N latents of 256 x 256 at C = 640 (84 MB per tensor and "
                         "latent), one JSON line per N with every kernel's effective GB/s")
    ap.add_argument("--pull-stitch", action="store_true", help="edge stitching as a separate halo gather (kernel mode 2) instead of the push fused into the normalisation")
    ap.add_argument("--library-yardstick", action="store_true",
                    help="instead of a configuration: the vendor libraries' bf16 GEMM (torch.matmul) and fused attention "
                         "(torch's scaled_dot_product_attention) on the shapes of configurations 2..5 with standard-normal operands, "
                         "one JSON line: a yardstick for the MFMA kernels, not part of the path")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true", help="do not bracket kernels with HIP events")
    ap.add_argument("--all-kernels", action="store_true", help="add every kernel's time and roofline fraction to the JSON")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2501_09253_amd as ps

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.pull_stitch:
        ps.set_kernel_mode(2)
    # one plain device copy of known size (256 MiB read + 256 MiB written): the reference that scales the
    # FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this same command
    cal_src = torch.ones(128 * 1024 * 1024, dtype=torch.bfloat16, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst
    peaks = None
    if not args.only:
        # what this chip reaches: a register-resident MFMA stream (about 30 ms) and a 2 GiB streaming copy
        big_src = torch.ones(1 << 30, dtype=torch.bfloat16, device="cuda")
        big_dst = torch.empty_like(big_src)
        # the matrix pipe's rate on constant operands (the datasheet's condition) and on standard-normal operands: the
        # chip lowers its clock with the bit activity of the data, so the second is what a real workload can reach
        const_tf, const_mhz = ps.probe_mfma_bf16(20000, False)
        rand_tf, rand_mhz = ps.probe_mfma_bf16(20000, True)
        # the same stream with the other instructions of a kernel's inner loop between the MFMAs (softmax work, LDS
        # fragment reads, row-sum MFMAs): the clock follows the power drawn, so this is the ceiling of that mix
        attn_tf, attn_mhz = ps.probe_mfma_mix(19, 20000)
        conv_tf, conv_mhz = ps.probe_mfma_mix(8, 20000)
        peaks = {"mfma_bf16_tflops": rand_tf, "mfma_bf16_mhz": rand_mhz, "mfma_bf16_constant_operands_tflops": const_tf,
                 "mfma_bf16_constant_operands_mhz": const_mhz, "attention_mix_tflops": attn_tf, "attention_mix_mhz": attn_mhz,
                 "conv_mix_tflops": conv_tf, "conv_mix_mhz": conv_mhz,
                 "copy_gbs": ps.probe_copy(big_dst, big_src, reps=5), "copy_bytes": 2 * big_src.numel()}
        del big_src, big_dst
        torch.cuda.empty_cache()

    if args.library_yardstick:
        print(json.dumps({"library_gemm": library_gemm(args.steps, args.warmup),
                          "library_attention": library_attention(min(args.steps, 5), min(max(1, args.warmup), 2)),
                          "measured_peaks": peaks}), flush=True)
        return

    if args.hbm_sweep:
        for n_images in args.hbm_sweep:
            r, _ = measure(0, args.steps, args.warmup, all_kernels=True, peaks=peaks, workload=big_workload(n_images))
            rows = {k: {"avg_us": v["avg_us"], "gbs": v["gbs"], "frac_hbm": v["frac_hbm"],
                        "frac_of_copy": None if peaks is None else v["gbs"] / peaks["copy_gbs"]}
                    for k, v in list(r["kernels"].items()) + list(r["extras"].items()) if "gbs" in v}
            print(json.dumps({"hbm_sweep": r["workload"], "tensor_MB": r["T"] * 640 * 2 / 1e6, "ms_per_step": r["ms_per_step"],
                              "copy_gbs": None if peaks is None else peaks["copy_gbs"], "kernels": rows}), flush=True)
        return

    events = not args.no_kernel_events
    res, w = measure(args.config, args.steps, args.warmup, all_kernels=args.all_kernels, events=events, patch=args.patch,
                     peaks=peaks)
    cpu = None if args.no_cpu_baseline else cpu_baseline(w)
    del w

    configs = None
    if not args.only:
        configs = []
        for c in (1, 2, 3, 4, 5):
            if c == args.config and args.patch is None:
                r = res
            else:
                r, _ = measure(c, min(args.steps, 20), min(args.warmup, 5), events=events, peaks=peaks)
            rf = r["roofline"] or {}
            configs.append({"workload": r["workload"], "ms_per_step": r["ms_per_step"], "tokens_per_s": r["tokens_per_s"],
                            "block_ms": r["block_ms"], "dominant_kernel": rf.get("kernel"), "bound": rf.get("bound"),
                            "kernel_avg_us": rf.get("avg_us"), "frac": rf.get("frac"),
                            "frac_of_measured": rf.get("frac_of_measured")})

    out = {
        "metric": "patch-tokens/sec per mixed-res denoising block", "value": res["tokens_per_s"],
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": res["dtype"], "data": "synthetic",
        "config": {"workload": res["workload"], "step": "split + block_forward + reassemble"},
        "block_forward_ms": res["block_ms"], "block_tokens_per_s": res["T"] / (res["block_ms"] * 1e-3), "plan_us": res["plan_us"],
        "computed_tokens": res["n_active"], "block_computed_tokens_per_s": res["n_active"] / (res["block_ms"] * 1e-3),
        "roofline": res["roofline"], "cpu_baseline": cpu, "measured_peaks": peaks, "configs": configs,
    }
    if args.all_kernels:
        out["kernels"] = res["kernels"]
        out["cache_manager"] = res["extras"]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
