"""Seeded synthetic inputs for the mixed-resolution patched denoising block.

This module only *draws numbers*: resolutions, latents, weights, text context,
cache slots and reuse masks of the five benchmark configurations.  It holds none
of the method's arithmetic (no normalisation, convolution, attention, patching),
so the CPU oracle and the HIP path can both be fed from it without sharing code.

Stand-in statement: the paper measures on SDXL / SD3 activations driven by
DiffusionDB and COCO prompts (Experiment section, "Workload").  Neither weights
nor prompts are available here, and the paper notes that performance does not
depend on the prompt, so seeded Gaussian tensors with the paper's *shapes*
(SDXL level widths 320/640/1280, latents of the 512/768/1024-pixel requests,
77 text tokens of width 2048) stand in for them.

Generator: SplitMix64 used as a counter-based generator (output k of a stream is
mix(seed + (k+1)*GAMMA)), 53-bit uniforms, Box-Muller normals.  Every tensor has
its own sub-stream keyed by (config seed, tensor name), so adding a tensor never
shifts the values of another one.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional, Tuple

import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_MASK64 = (1 << 64) - 1

BASE_SEED = 0x5EED0000


def _mix64(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _fnv1a(name: str) -> int:
    h = 0xCBF29CE484222325
    for b in name.encode():
        h = ((h ^ b) * 0x100000001B3) & _MASK64
    return h


class Stream:
    """One counter-based SplitMix64 stream."""

    def __init__(self, seed: int, name: str = ""):
        s = (int(seed) ^ _fnv1a(name)) & _MASK64
        # one scalar mixing round decorrelates neighbouring seeds / names
        self._seed = int(_mix64(np.array([s], dtype=np.uint64))[0])
        self._pos = 0

    def raw(self, count: int) -> np.ndarray:
        with np.errstate(over="ignore"):
            k = np.arange(self._pos + 1, self._pos + count + 1, dtype=np.uint64)
            z = np.uint64(self._seed) + k * _GAMMA
            out = _mix64(z)
        self._pos += count
        return out

    def uniform(self, count: int) -> np.ndarray:
        """count doubles in [0, 1)."""
        return (self.raw(count) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))

    def randint(self, count: int, k: int) -> np.ndarray:
        return np.minimum((self.uniform(count) * k).astype(np.int64), k - 1)

    def normal(self, shape, chunk: int = 1 << 22) -> np.ndarray:
        """Standard normals as float32 (Box-Muller on consecutive uniform pairs)."""
        total = int(np.prod(shape)) if len(tuple(np.atleast_1d(shape))) else 1
        out = np.empty(total, dtype=np.float32)
        chunk = max(2, chunk & ~1)          # whole Box-Muller pairs per chunk
        done = 0
        while done < total:
            m = min(chunk, total - done)
            pairs = (m + 1) // 2
            u = self.uniform(2 * pairs)
            u1 = 1.0 - u[0::2]                      # (0, 1]
            r = np.sqrt(-2.0 * np.log(u1))
            th = (2.0 * math.pi) * u[1::2]
            z = np.empty(2 * pairs, dtype=np.float64)
            z[0::2] = r * np.cos(th)
            z[1::2] = r * np.sin(th)
            out[done:done + m] = z[:m].astype(np.float32)
            done += m
        return out.reshape(shape)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    b = x.view(np.uint32)
    lsb = (b >> np.uint32(16)) & np.uint32(1)
    r = (b + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32).reshape(x.shape)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """bf16-representable float32 values -> their 16-bit patterns (uint16)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16).reshape(x.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).reshape(b.shape)


# stage names of the block grammar
RES1, RES2, SATTN, XATTN, FFN = "RES1", "RES2", "SATTN", "XATTN", "FFN"
# the same three with a per-pixel LayerNorm in front (transformer layer of an SDXL level)
LSATTN, LXATTN, LFFN = "LSATTN", "LXATTN", "LFFN"
# RES2 with the per-request time embedding added after the first convolution (residual block of an SDXL level)
RES2T = "RES2T"
# sub-layers of a diffusion-transformer block: adaptive LayerNorm modulation from the per-request vector, gated residual
ASATTN, AMLP = "ASATTN", "AMLP"
# a whole joint text-image block of that model (needs a joint plan: ctx_len text tokens of width C per request)
MMDIT = "MMDIT"


@dataclasses.dataclass
class Config:
    cfg_id: int
    name: str
    dtype: str                       # "f32" | "bf16"
    resolutions: List[Tuple[int, int]]   # latent (H, W) per request, caller order
    patch: Tuple[int, int]
    C: int
    G: int
    heads: int
    d: int
    stages: Tuple[str, ...]
    ctx_len: int = 0
    ctx_dim: int = 0
    ffn_mult: int = 4
    reuse_p: float = 0.0
    eps: float = 1e-5
    seed: int = 0
    temb_dim: int = 0                # width of the per-request time embedding (RES2T), else 0

    @property
    def n(self) -> int:
        return len(self.resolutions)

    @property
    def grids(self) -> List[Tuple[int, int]]:
        return [(h // self.patch[0], w // self.patch[1]) for h, w in self.resolutions]

    @property
    def P(self) -> int:
        return sum(a * b for a, b in self.grids)

    @property
    def T(self) -> int:
        return sum(h * w for h, w in self.resolutions)


def _draw_res(seed: int, n: int, sizes) -> List[Tuple[int, int]]:
    idx = Stream(seed, "resolutions").randint(n, len(sizes))
    return [(sizes[i], sizes[i]) for i in idx]


def config(cfg_id: int, seed: Optional[int] = None) -> Config:
    """The five benchmark configurations (resolutions of 3 and 4 are drawn from the seed)."""
    s = BASE_SEED + cfg_id if seed is None else seed
    if cfg_id == 1:
        return Config(1, "tiny-fp32", "f32", [(16, 16), (24, 24)], (8, 8), 64, 8, 2, 32,
                      (RES1, SATTN), seed=s)
    if cfg_id == 2:
        return Config(2, "sdxl-resnet-c320", "bf16", [(64, 64), (96, 96), (128, 128)], (32, 32),
                      320, 32, 5, 64, (RES2,), seed=s)
    if cfg_id == 3:
        return Config(3, "sdxl-transformer-c640", "bf16", _draw_res(s, 8, (32, 48, 64)), (16, 16),
                      640, 32, 10, 64, (SATTN, XATTN, FFN), ctx_len=77, ctx_dim=2048, seed=s)
    if cfg_id == 4:
        return Config(4, "sdxl-mid-c1280", "bf16", _draw_res(s, 24, (16, 24, 32)), (8, 8),
                      1280, 32, 20, 64, (RES2, SATTN, XATTN), ctx_len=77, ctx_dim=2048, seed=s)
    if cfg_id == 5:
        return Config(5, "skewed-reuse-c640", "bf16", [(256, 256)] + [(64, 64)] * 16, (32, 32),
                      640, 32, 10, 64, (RES2, SATTN), reuse_p=0.4, seed=s)
    if cfg_id == 6:      # config 3 as a transformer layer with per-pixel LayerNorms (not a configuration of the baseline list)
        return Config(6, "sdxl-transformer-ln-c640", "bf16", _draw_res(BASE_SEED + 3 if seed is None else seed, 8, (32, 48, 64)),
                      (16, 16), 640, 32, 10, 64, (LSATTN, LXATTN, LFFN), ctx_len=77, ctx_dim=2048, seed=s)
    if cfg_id == 9:      # a joint text-image block at the second model's width, 154 text tokens per request; not in the baseline list
        return Config(9, "mmdit-block-c1536", "bf16", [(32, 32), (48, 48), (64, 64), (64, 64)], (16, 16),
                      1536, 32, 24, 64, (MMDIT,), ctx_len=154, ctx_dim=1536, seed=s, temb_dim=1536)
    if cfg_id == 8:      # a diffusion-transformer block (adaLN sub-layers) at the second model's width; not in the baseline list
        return Config(8, "dit-block-c1536", "bf16", [(32, 32), (48, 48), (64, 64), (64, 64)], (16, 16),
                      1536, 32, 24, 64, (ASATTN, AMLP), seed=s, temb_dim=1536)
    if cfg_id == 7:      # config 2 with the time embedding (SDXL: 1280 wide); not a configuration of the baseline list
        return Config(7, "sdxl-resnet-temb-c320", "bf16", [(64, 64), (96, 96), (128, 128)], (32, 32),
                      320, 32, 5, 64, (RES2T,), seed=s, temb_dim=1280)
    raise ValueError(f"unknown config {cfg_id}")


def custom_config(resolutions, patch, C, G, heads, stages, dtype="f32", ctx_len=0, ctx_dim=0,
                  reuse_p=0.0, seed=1234, ffn_mult=4, temb_dim=0) -> Config:
    """A free-form configuration for edge-case tests."""
    return Config(0, "custom", dtype, [tuple(r) for r in resolutions], tuple(patch), C, G, heads,
                  C // heads, tuple(stages), ctx_len=ctx_len, ctx_dim=ctx_dim, reuse_p=reuse_p,
                  seed=seed, ffn_mult=ffn_mult, temb_dim=temb_dim)


# parameter shapes per stage type: name -> (shape builder, kind)
def stage_param_shapes(stage: str, cfg: Config) -> Dict[str, Tuple[Tuple[int, ...], str]]:
    C = cfg.C
    F = cfg.ffn_mult * C
    if stage == RES1:
        return {"gn_g": ((C,), "gamma"), "gn_b": ((C,), "beta"),
                "conv_w": ((C, C, 3, 3), "w:%d" % (9 * C)), "conv_b": ((C,), "bias")}
    if stage == RES2:
        return {"gn_a_g": ((C,), "gamma"), "gn_a_b": ((C,), "beta"),
                "conv_a_w": ((C, C, 3, 3), "w:%d" % (9 * C)), "conv_a_b": ((C,), "bias"),
                "gn_b_g": ((C,), "gamma"), "gn_b_b": ((C,), "beta"),
                "conv_b_w": ((C, C, 3, 3), "w:%d" % (9 * C)), "conv_b_b": ((C,), "bias")}
    if stage == RES2T:
        D = cfg.temb_dim
        return {**stage_param_shapes(RES2, cfg), "wt": ((D, C), "w:%d" % D), "bt": ((C,), "bias")}
    if stage == SATTN:
        return {"gn_g": ((C,), "gamma"), "gn_b": ((C,), "beta"),
                "wq": ((C, C), "w:%d" % C), "wk": ((C, C), "w:%d" % C), "wv": ((C, C), "w:%d" % C),
                "wo": ((C, C), "w:%d" % C), "bo": ((C,), "bias")}
    if stage == XATTN:
        D = cfg.ctx_dim
        return {"wq": ((C, C), "w:%d" % C), "wk": ((D, C), "w:%d" % D), "wv": ((D, C), "w:%d" % D),
                "wo": ((C, C), "w:%d" % C), "bo": ((C,), "bias")}
    if stage == FFN:
        return {"w1": ((C, 2 * F), "w:%d" % C), "b1": ((2 * F,), "bias"),
                "w2": ((F, C), "w:%d" % F), "b2": ((C,), "bias")}
    if stage == MMDIT:
        D = cfg.temb_dim
        one = {"wm": ((D, 6 * C), "w:%d" % D), "bm": ((6 * C,), "bias"),
               "wq": ((C, C), "w:%d" % C), "wk": ((C, C), "w:%d" % C), "wv": ((C, C), "w:%d" % C),
               "wo": ((C, C), "w:%d" % C), "bo": ((C,), "bias"),
               "w1": ((C, F), "w:%d" % C), "b1": ((F,), "bias"), "w2": ((F, C), "w:%d" % F), "b2": ((C,), "bias")}
        return {X + "." + k: v for X in ("img", "txt") for k, v in one.items()}
    if stage == ASATTN:
        D = cfg.temb_dim
        return {"wm": ((D, 3 * C), "w:%d" % D), "bm": ((3 * C,), "bias"),
                "wq": ((C, C), "w:%d" % C), "wk": ((C, C), "w:%d" % C), "wv": ((C, C), "w:%d" % C),
                "wo": ((C, C), "w:%d" % C), "bo": ((C,), "bias")}
    if stage == AMLP:
        D = cfg.temb_dim
        return {"wm": ((D, 3 * C), "w:%d" % D), "bm": ((3 * C,), "bias"),
                "w1": ((C, F), "w:%d" % C), "b1": ((F,), "bias"), "w2": ((F, C), "w:%d" % F), "b2": ((C,), "bias")}
    if stage in (LSATTN, LXATTN, LFFN):
        base = stage_param_shapes(stage[1:], cfg)
        base.pop("gn_g", None)
        base.pop("gn_b", None)
        return {"ln_g": ((C,), "gamma"), "ln_b": ((C,), "beta"), **base}
    raise ValueError(stage)


def stage_cache_slots(stage: str) -> Tuple[str, ...]:
    """Names of the cached operand tensors a stage keeps for reused patches."""
    if stage in (RES2, RES2T):
        return ("h1",)
    if stage == SATTN:
        return ("r", "K", "V")
    if stage in (LSATTN, ASATTN):
        return ("K", "V")
    return ()


@dataclasses.dataclass
class Workload:
    cfg: Config
    images: List[np.ndarray]                  # per request [C, H, W] float32, caller order
    params: List[Dict[str, np.ndarray]]       # per stage
    ctx: Optional[np.ndarray]                 # [n, ctx_len, ctx_dim] float32 or None
    reuse: Optional[List[np.ndarray]]         # per request bool [gh, gw] (True = reuse) or None
    cache: Optional[Dict[str, List[np.ndarray]]]  # slot name -> per request [C, H, W] float32
    temb: Optional[np.ndarray] = None         # [n, temb_dim] float32 or None


def make_workload(cfg: Config) -> Workload:
    """Draw every tensor of a configuration.  bf16 configurations hold bf16-representable float32."""
    rd = bf16_round if cfg.dtype == "bf16" else (lambda a: a)
    seed = cfg.seed
    images = [rd(Stream(seed, f"image{i}").normal((cfg.C, h, w)))
              for i, (h, w) in enumerate(cfg.resolutions)]
    params = []
    for si, st in enumerate(cfg.stages):
        d = {}
        for name, (shape, kind) in stage_param_shapes(st, cfg).items():
            z = Stream(seed, f"stage{si}.{name}").normal(shape)
            if kind == "gamma":
                z = 1.0 + 0.1 * z
            elif kind in ("beta", "bias"):
                z = 0.1 * z
            else:
                fan_in = int(kind.split(":")[1])
                z = z * np.float32(1.0 / math.sqrt(fan_in))
            d[name] = rd(z.astype(np.float32))
        params.append(d)
    ctx = None
    if cfg.ctx_len:
        ctx = rd(Stream(seed, "ctx").normal((cfg.n, cfg.ctx_len, cfg.ctx_dim)))
    reuse = cache = None
    if cfg.reuse_p > 0.0:
        reuse = []
        for i, (gh, gw) in enumerate(cfg.grids):
            u = Stream(seed, f"reuse{i}").uniform(gh * gw)
            reuse.append((u < cfg.reuse_p).reshape(gh, gw))
        cache = {}
        names = [f"{si}.{sl}" for si, st in enumerate(cfg.stages) for sl in stage_cache_slots(st)]
        for nm in names + ["y"]:
            cache[nm] = [rd(Stream(seed, f"cache.{nm}.{i}").normal((cfg.C, h, w)))
                         for i, (h, w) in enumerate(cfg.resolutions)]
    temb = rd(Stream(seed, "temb").normal((cfg.n, cfg.temb_dim))) if cfg.temb_dim else None
    return Workload(cfg, images, params, ctx, reuse, cache, temb)
