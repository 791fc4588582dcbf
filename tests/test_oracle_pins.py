"""Pins of the CPU oracle against things other than itself (CPU only).

Each check is chosen so that one plausible mistake in the oracle (dropped term,
wrong sign or index, transposed operand, wrong padding, wrong group layout)
fails it: brute-force loops on tiny inputs, closed forms, invariants, printed
constants and independent torch CPU library routines.
"""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads as wl
from oracle import block as ob
from oracle import plan as op
from oracle import cache as oc
from oracle import resample as orr
from oracle import sched as osc

RNG = np.random.default_rng(7)


# ----------------------------------------------------------------------------- pointwise
def test_silu_gelu_constants():
    assert abs(ob.silu(np.array([1.0]))[0] - 0.7310585786300049) < 1e-15
    assert abs(ob.gelu(np.array([1.0]))[0] - 0.8413447460685429) < 1e-15
    assert ob.gelu(np.array([0.0]))[0] == 0.0 and ob.silu(np.array([0.0]))[0] == 0.0
    # odd/even structure: silu(u) - silu(-u) = u, gelu(u) - gelu(-u) = u
    u = RNG.standard_normal(100)
    assert np.allclose(ob.silu(u) - ob.silu(-u), u, atol=1e-14)
    assert np.allclose(ob.gelu(u) - ob.gelu(-u), u, atol=1e-14)
    assert np.allclose(ob.gelu(u), F.gelu(torch.from_numpy(u)).numpy(), atol=1e-14)
    assert np.allclose(ob.silu(u), F.silu(torch.from_numpy(u)).numpy(), atol=1e-14)


# ----------------------------------------------------------------------------- conv3
def _conv_loops(u, W, b):
    Ci, H, Wd = u.shape
    Co = W.shape[0]
    out = np.zeros((Co, H, Wd))
    for co in range(Co):
        for y in range(H):
            for x in range(Wd):
                acc = b[co]
                for ci in range(Ci):
                    for ky in range(3):
                        for kx in range(3):
                            yy, xx = y + ky - 1, x + kx - 1
                            if 0 <= yy < H and 0 <= xx < Wd:
                                acc += u[ci, yy, xx] * W[co, ci, ky, kx]
                out[co, y, x] = acc
    return out


def test_conv3_vs_seven_loops():
    u = RNG.standard_normal((3, 5, 4))
    W = RNG.standard_normal((2, 3, 3, 3))
    b = RNG.standard_normal(2)
    assert np.allclose(ob.conv3(u, W, b), _conv_loops(u, W, b), atol=1e-13)


def test_conv3_delta_kernel_is_identity_plus_bias():
    C = 4
    u = RNG.standard_normal((C, 6, 7))
    W = np.zeros((C, C, 3, 3))
    W[np.arange(C), np.arange(C), 1, 1] = 1.0
    b = RNG.standard_normal(C)
    assert np.allclose(ob.conv3(u, W, b), u + b[:, None, None], atol=1e-15)


def test_conv3_single_off_centre_tap_shifts_the_right_way():
    # only W[0,0,ky=0,kx=2] = 1: out[y,x] = u[y-1, x+1] (cross-correlation, not flipped)
    u = RNG.standard_normal((1, 5, 6))
    W = np.zeros((1, 1, 3, 3))
    W[0, 0, 0, 2] = 1.0
    out = ob.conv3(u, W, np.zeros(1))
    exp = np.zeros_like(u)
    exp[0, 1:, :-1] = u[0, :-1, 1:]
    assert np.array_equal(out, exp)


def test_conv3_channel_operand_not_transposed():
    # W[co=1, ci=0] centre tap only: output channel 1 = input channel 0, output channel 0 = 0
    u = RNG.standard_normal((2, 4, 4))
    W = np.zeros((2, 2, 3, 3))
    W[1, 0, 1, 1] = 1.0
    out = ob.conv3(u, W, np.zeros(2))
    assert np.array_equal(out[1], u[0]) and not out[0].any()


def test_conv3_all_ones_closed_form_pins_zero_padding():
    Ci, H, Wd, c = 3, 5, 6, 0.5
    out = ob.conv3(np.full((Ci, H, Wd), c), np.ones((2, Ci, 3, 3)), np.zeros(2))
    assert np.allclose(out[:, 1:-1, 1:-1], 9 * Ci * c)
    assert np.allclose(out[:, 0, 1:-1], 6 * Ci * c) and np.allclose(out[:, 1:-1, -1], 6 * Ci * c)
    for yy, xx in [(0, 0), (0, -1), (-1, 0), (-1, -1)]:
        assert np.allclose(out[:, yy, xx], 4 * Ci * c)


def test_conv3_vs_torch_library():
    u = RNG.standard_normal((5, 9, 7))
    W = RNG.standard_normal((4, 5, 3, 3))
    b = RNG.standard_normal(4)
    ref = F.conv2d(torch.from_numpy(u)[None], torch.from_numpy(W), torch.from_numpy(b), padding=1)[0].numpy()
    assert np.allclose(ob.conv3(u, W, b), ref, atol=1e-12)


# ----------------------------------------------------------------------------- GroupNorm
def test_group_norm_moments_and_group_layout():
    C, G, H, W, eps = 12, 3, 5, 6, 1e-5
    # every channel gets its own offset so that a wrong channel->group mapping changes the moments
    u = RNG.standard_normal((C, H, W)) * (1 + np.arange(C))[:, None, None] + 3 * np.arange(C)[:, None, None]
    y = ob.group_norm(u, np.ones(C), np.zeros(C), G, eps)
    cg = C // G
    for g in range(G):
        blk, src = y[g * cg:(g + 1) * cg], u[g * cg:(g + 1) * cg]
        var = src.var()
        assert abs(blk.mean()) < 1e-12
        assert abs(blk.var() - var / (var + eps)) < 1e-12


def test_group_norm_shift_scale_invariance_and_affine():
    C, G, eps = 8, 2, 1e-5
    u = RNG.standard_normal((C, 4, 4))
    gam, bet = RNG.standard_normal(C), RNG.standard_normal(C)
    y0 = ob.group_norm(u, gam, bet, G, 0.0)
    y1 = ob.group_norm(5.0 * u + 11.0, gam, bet, G, 0.0)
    assert np.allclose(y0, y1, atol=1e-10)
    # affine is per channel: (y - beta)/gamma is the plain normalised tensor
    yn = ob.group_norm(u, np.ones(C), np.zeros(C), G, eps)
    ya = ob.group_norm(u, gam, bet, G, eps)
    assert np.allclose(ya, yn * gam[:, None, None] + bet[:, None, None], atol=1e-14)


def test_group_norm_vs_torch_library():
    C, G = 20, 4
    u = RNG.standard_normal((C, 7, 5)) + 2.0
    gam, bet = RNG.standard_normal(C), RNG.standard_normal(C)
    ref = F.group_norm(torch.from_numpy(u)[None], G, torch.from_numpy(gam), torch.from_numpy(bet), 1e-5)[0].numpy()
    assert np.allclose(ob.group_norm(u, gam, bet, G, 1e-5), ref, atol=1e-12)


# ----------------------------------------------------------------------------- attention
def _attn_three_pass(Q, K, V, heads):
    Nq, C = Q.shape
    d = C // heads
    out = np.zeros((Nq, C))
    for h in range(heads):
        for i in range(Nq):
            s = [sum(Q[i, h * d + c] * K[j, h * d + c] for c in range(d)) / math.sqrt(d) for j in range(K.shape[0])]
            m = max(s)
            e = [math.exp(v - m) for v in s]
            z = sum(e)
            for c in range(d):
                out[i, h * d + c] = sum(e[j] / z * V[j, h * d + c] for j in range(K.shape[0]))
    return out


def test_layer_norm_closed_forms():
    """Channels (1, 2, 3, 4): mean 5/2, biased variance 5/4, so with eps = 0 the result is (-3, -1, 1, 3) / sqrt 5;
    a pixel whose channels are all equal gives beta exactly; each pixel is normalised on its own."""
    u = np.zeros((4, 2, 3))
    u[:, 0, 0] = [1, 2, 3, 4]
    u[:, 1, 2] = 7.0
    u[:, 0, 1] = [10, 20, 30, 40]                                   # a multiple: same normalised values
    one, zero = np.ones(4), np.zeros(4)
    y = ob.layer_norm(u, one, zero, 0.0 + 1e-300)
    want = np.array([-3, -1, 1, 3]) / math.sqrt(5.0)
    assert np.allclose(y[:, 0, 0], want, atol=1e-14) and np.allclose(y[:, 0, 1], want, atol=1e-14)
    g, b = np.array([2.0, -1.0, 0.5, 3.0]), np.array([0.1, 0.2, 0.3, 0.4])
    y = ob.layer_norm(u, g, b, 1e-5)
    assert np.array_equal(y[:, 1, 2], b)                           # zero variance: only the shift is left
    assert np.allclose(y[:, 0, 0], want * g * math.sqrt(1.25 / (1.25 + 1e-5)) + b, atol=1e-14)
    # the channel axis is the one reduced: per-pixel mean 0 and variance var / (var + eps) before the affine map
    z = wl.Stream(7, "ln").normal((6, 3, 5)).astype(np.float64)
    n = ob.layer_norm(z, np.ones(6), np.zeros(6), 1e-5)
    assert np.allclose(n.mean(axis=0), 0.0, atol=1e-14)
    v = z.var(axis=0)
    assert np.allclose(n.var(axis=0), v / (v + 1e-5), atol=1e-12)


def test_layer_norm_vs_torch_library():
    z = wl.Stream(8, "ln").normal((12, 4, 6)).astype(np.float64)
    g, b = wl.Stream(8, "g").normal((12,)).astype(np.float64), wl.Stream(8, "b").normal((12,)).astype(np.float64)
    ref = F.layer_norm(torch.from_numpy(z).permute(1, 2, 0), (12,), torch.from_numpy(g), torch.from_numpy(b), 1e-5)
    assert np.allclose(ob.layer_norm(z, g, b, 1e-5), ref.permute(2, 0, 1).numpy(), atol=1e-12)


def test_l_stages_act_per_pixel_where_they_should():
    """LXATTN and LFFN see one pixel at a time: a crop of the input gives the crop of the output (so patching cannot
    change them); LSATTN mixes the pixels of an image: the same crop test must fail for it."""
    cfg = wl.custom_config([(6, 8)], (2, 2), C=16, G=4, heads=2, stages=(wl.LXATTN, wl.LFFN), ctx_len=5, ctx_dim=12, seed=17)
    w = wl.make_workload(cfg)
    z = w.images[0]
    full, _ = ob.block_forward(z, cfg.stages, w.params, G=cfg.G, heads=cfg.heads, ctx=w.ctx[0])
    crop, _ = ob.block_forward(z[:, 2:4, 3:7], cfg.stages, w.params, G=cfg.G, heads=cfg.heads, ctx=w.ctx[0])
    assert np.allclose(crop, full[:, 2:4, 3:7], atol=1e-13)
    cfg2 = wl.custom_config([(6, 8)], (2, 2), C=16, G=4, heads=2, stages=(wl.LSATTN,), seed=17)
    w2 = wl.make_workload(cfg2)
    full2, _ = ob.block_forward(z, cfg2.stages, w2.params, G=cfg2.G, heads=cfg2.heads)
    crop2, _ = ob.block_forward(z[:, 2:4, 3:7], cfg2.stages, w2.params, G=cfg2.G, heads=cfg2.heads)
    assert np.abs(crop2 - full2[:, 2:4, 3:7]).max() > 1e-3


def test_lsattn_reuse_follows_operand_fill_rule():
    """Mixed reuse through LSATTN with torch pieces: K and V of reused patches are the cached ones, queries and the
    residual of computed patches are fresh, reused patches of the output are the cached output."""
    cfg = wl.custom_config([(8, 8), (4, 8)], (4, 4), C=8, G=2, heads=2, stages=(wl.LSATTN, wl.LFFN), reuse_p=0.5, seed=3)
    w = wl.make_workload(cfg)
    assert set(w.cache) == {"0.K", "0.V", "y"}
    y, nc = ob.forward_batch(w.images, cfg.stages, w.params, G=cfg.G, heads=cfg.heads, reuse=w.reuse, cache=w.cache)
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    ph, pw = cfg.patch
    for i, z in enumerate(w.images):
        C, H, W = z.shape
        m = t(np.kron(w.reuse[i].astype(np.float64), np.ones((ph, pw)))).bool()
        mt = m.reshape(-1, 1)
        p0, p1 = w.params
        xt = t(z).flatten(1).T
        u = F.layer_norm(xt, (C,), t(p0["ln_g"]), t(p0["ln_b"]), cfg.eps)
        k = torch.where(mt, t(w.cache["0.K"][i]).flatten(1).T, u @ t(p0["wk"]))
        v = torch.where(mt, t(w.cache["0.V"][i]).flatten(1).T, u @ t(p0["wv"]))
        sp = lambda a: a.reshape(1, -1, cfg.heads, C // cfg.heads).transpose(1, 2)
        o = F.scaled_dot_product_attention(sp(u @ t(p0["wq"])), sp(k), sp(v)).transpose(1, 2).reshape(-1, C)
        r = xt + o @ t(p0["wo"]) + t(p0["bo"])
        a, g = (F.layer_norm(r, (C,), t(p1["ln_g"]), t(p1["ln_b"]), cfg.eps) @ t(p1["w1"]) + t(p1["b1"])).chunk(2, dim=-1)
        out = r + (a * F.gelu(g)) @ t(p1["w2"]) + t(p1["b2"])
        out = torch.where(mt, t(w.cache["y"][i]).flatten(1).T, out).T.reshape(C, H, W).numpy()
        mm = m.numpy()
        # computed patches only: a reused patch's fresh values are never formed by the method
        assert np.allclose(y[i][:, ~mm], out[:, ~mm], atol=1e-10)
        assert np.array_equal(y[i][:, mm], w.cache["y"][i].astype(np.float64)[:, mm])
        assert np.allclose(nc[i]["0.K"], k.T.reshape(C, H, W).numpy(), atol=1e-10)


def test_res2t_time_embedding_closed_forms():
    """W_t = 0, b_t = 0 gives RES2; a zero embedding adds b_t alone (SiLU(0) = 0); the added term is the same for every
    pixel of a request and differs between requests: with conv_a = 0 the first convolution's output is the term itself
    (slot h1 under an all-compute mask), e = SiLU(temb) W_t + b_t computed here by a plain loop."""
    cfg = wl.custom_config([(4, 6), (4, 4)], (2, 2), C=8, G=2, heads=1, stages=(wl.RES2T,), seed=12, temb_dim=5)
    w = wl.make_workload(cfg)
    p = dict(w.params[0])
    kw = dict(G=cfg.G, heads=cfg.heads, eps=cfg.eps)
    plain, _ = ob.forward_batch(w.images, (wl.RES2,), [p], **kw)
    p0 = dict(p, wt=np.zeros_like(p["wt"]), bt=np.zeros_like(p["bt"]))
    y0, _ = ob.forward_batch(w.images, cfg.stages, [p0], temb=w.temb, **kw)
    for a, b in zip(plain, y0):
        assert np.array_equal(a, b)
    pz = dict(p, conv_a_w=np.zeros_like(p["conv_a_w"]), conv_a_b=np.zeros_like(p["conv_a_b"]))
    none = [np.zeros((h // 2, w_ // 2), dtype=bool) for h, w_ in cfg.resolutions]
    dummy = {"0.h1": [np.zeros_like(z) for z in w.images], "y": [np.zeros_like(z) for z in w.images]}
    _, nc = ob.forward_batch(w.images, cfg.stages, [pz], temb=w.temb, reuse=none, cache=dummy, **kw)
    for i in range(cfg.n):
        e = np.zeros(8)
        for c in range(8):
            acc = float(p["bt"][c])
            for k in range(5):
                tk = float(w.temb[i][k])
                acc += tk / (1.0 + math.exp(-tk)) * float(p["wt"][k, c])
            e[c] = acc
        assert np.allclose(nc[i]["0.h1"], np.broadcast_to(e[:, None, None], w.images[i].shape), atol=1e-13)
    _, ncz = ob.forward_batch(w.images, cfg.stages, [pz], temb=np.zeros_like(w.temb), reuse=none, cache=dummy, **kw)
    assert np.allclose(ncz[0]["0.h1"], np.broadcast_to(p["bt"].astype(np.float64)[:, None, None], w.images[0].shape), atol=1e-15)


def test_adaln_closed_forms():
    """W_m = 0 with b_m = (0, 0, gate): the modulation is the identity on LN0(x), the sub-layer output is scaled by the
    gate; gate 0 returns x exactly (the zero-initialised form); GELU tanh form at 1: 0.5 (1 + tanh(sqrt(2/pi) 1.044715))."""
    assert abs(float(ob.gelu_tanh(np.array(1.0))) - 0.5 * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * 1.044715))) < 1e-15
    assert abs(float(ob.gelu_tanh(np.array(1.0))) - 0.8411919906082768) < 1e-12
    cfg = wl.custom_config([(4, 6)], (2, 2), C=8, G=1, heads=2, stages=(wl.AMLP,), seed=14, temb_dim=5, ffn_mult=2)
    w = wl.make_workload(cfg)
    p = dict(w.params[0])
    kw = dict(G=cfg.G, heads=cfg.heads, eps=cfg.eps)
    z = w.images[0].astype(np.float64)
    bm = np.zeros(24)
    p0 = dict(p, wm=np.zeros_like(p["wm"]), bm=bm)
    y0, _ = ob.block_forward(z, cfg.stages, [p0], temb=w.temb[0], **kw)
    assert np.array_equal(y0, z)                                       # gate 0
    bm1 = bm.copy()
    bm1[16:] = 2.0
    y1, _ = ob.block_forward(z, cfg.stages, [dict(p0, bm=bm1)], temb=w.temb[0], **kw)
    xt = z.reshape(8, -1).T
    xh = (xt - xt.mean(1, keepdims=True)) / np.sqrt(xt.var(1, keepdims=True) + cfg.eps)
    d = ob.gelu_tanh(xh @ p["w1"].astype(np.float64) + p["b1"]) @ p["w2"].astype(np.float64) + p["b2"]
    assert np.allclose(y1, (xt + 2.0 * d).T.reshape(z.shape), atol=1e-12)
    bm2 = bm1.copy()
    bm2[:8] = 0.5                                                      # shift 0.5
    bm2[8:16] = 1.0                                                    # scale 1: h = 2 LN0(x) + 0.5
    y2, _ = ob.block_forward(z, cfg.stages, [dict(p0, bm=bm2)], temb=w.temb[0], **kw)
    d2 = ob.gelu_tanh((2.0 * xh + 0.5) @ p["w1"].astype(np.float64) + p["b1"]) @ p["w2"].astype(np.float64) + p["b2"]
    assert np.allclose(y2, (xt + 2.0 * d2).T.reshape(z.shape), atol=1e-12)


def test_attention_vs_three_pass_loops():
    Q, K, V = RNG.standard_normal((5, 6)), RNG.standard_normal((7, 6)), RNG.standard_normal((7, 6))
    assert np.allclose(ob.attention(Q, K, V, 2), _attn_three_pass(Q, K, V, 2), atol=1e-13)
    rows = np.array([4, 1])
    assert np.allclose(ob.attention(Q, K, V, 2, rows=rows), _attn_three_pass(Q, K, V, 2)[rows], atol=1e-13)


def test_attention_zero_queries_give_mean_of_values():
    K, V = RNG.standard_normal((9, 8)), RNG.standard_normal((9, 8))
    out = ob.attention(np.zeros((4, 8)), K, V, 2)
    assert np.allclose(out, np.broadcast_to(V.mean(axis=0), (4, 8)), atol=1e-14)


def test_attention_permutation_equivariance_and_chunking():
    Q, K, V = RNG.standard_normal((10, 8)), RNG.standard_normal((10, 8)), RNG.standard_normal((10, 8))
    base = ob.attention(Q, K, V, 2)
    pk = RNG.permutation(10)
    assert np.allclose(ob.attention(Q, K[pk], V[pk], 2), base, atol=1e-13)       # key order is irrelevant
    pq = RNG.permutation(10)
    assert np.allclose(ob.attention(Q[pq], K, V, 2), base[pq], atol=1e-13)       # query rows are independent
    assert np.allclose(ob.attention(Q, K, V, 2, chunk=3), base, atol=1e-14)


def test_attention_vs_torch_library():
    N, heads, d = 11, 3, 4
    Q, K, V = (RNG.standard_normal((N, heads * d)) for _ in range(3))
    def th(a):
        return torch.from_numpy(a).reshape(N, heads, d).permute(1, 0, 2)[None]
    ref = F.scaled_dot_product_attention(th(Q), th(K), th(V))[0].permute(1, 0, 2).reshape(N, heads * d).numpy()
    assert np.allclose(ob.attention(Q, K, V, heads), ref, atol=1e-12)


# ----------------------------------------------------------------------------- whole block vs torch composition
def _torch_block(z, cfg, params, ctx, temb=None):
    """The block grammar composed from torch CPU library routines in float64 (independent of the oracle)."""
    x = torch.from_numpy(np.asarray(z, dtype=np.float64))[None]
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    C, H, W = z.shape
    hd = cfg.heads

    def mha(q, k, v):
        q = q.reshape(1, -1, hd, C // hd).transpose(1, 2)
        k = k.reshape(1, -1, hd, C // hd).transpose(1, 2)
        v = v.reshape(1, -1, hd, C // hd).transpose(1, 2)
        return F.scaled_dot_product_attention(q, k, v).transpose(1, 2).reshape(1, -1, C)

    for st, p in zip(cfg.stages, params):
        if st == wl.RES1:
            x = x + F.conv2d(F.silu(F.group_norm(x, cfg.G, t(p["gn_g"]), t(p["gn_b"]), cfg.eps)),
                             t(p["conv_w"]), t(p["conv_b"]), padding=1)
        elif st == wl.RES2:
            h = F.conv2d(F.silu(F.group_norm(x, cfg.G, t(p["gn_a_g"]), t(p["gn_a_b"]), cfg.eps)),
                         t(p["conv_a_w"]), t(p["conv_a_b"]), padding=1)
            x = x + F.conv2d(F.silu(F.group_norm(h, cfg.G, t(p["gn_b_g"]), t(p["gn_b_b"]), cfg.eps)),
                             t(p["conv_b_w"]), t(p["conv_b_b"]), padding=1)
        elif st == wl.RES2T:
            e = F.linear(F.silu(t(temb)), t(p["wt"]).T, t(p["bt"]))
            h = F.conv2d(F.silu(F.group_norm(x, cfg.G, t(p["gn_a_g"]), t(p["gn_a_b"]), cfg.eps)),
                         t(p["conv_a_w"]), t(p["conv_a_b"]), padding=1) + e[None, :, None, None]
            x = x + F.conv2d(F.silu(F.group_norm(h, cfg.G, t(p["gn_b_g"]), t(p["gn_b_b"]), cfg.eps)),
                             t(p["conv_b_w"]), t(p["conv_b_b"]), padding=1)
        elif st == wl.SATTN:
            u = F.group_norm(x, cfg.G, t(p["gn_g"]), t(p["gn_b"]), cfg.eps).flatten(2).transpose(1, 2)
            o = mha(u @ t(p["wq"]), u @ t(p["wk"]), u @ t(p["wv"]))
            x = x + (o @ t(p["wo"]) + t(p["bo"])).transpose(1, 2).reshape(1, C, H, W)
        elif st == wl.XATTN:
            xt = x.flatten(2).transpose(1, 2)
            c = t(ctx)[None]
            o = mha(xt @ t(p["wq"]), c @ t(p["wk"]), c @ t(p["wv"]))
            x = (xt + o @ t(p["wo"]) + t(p["bo"])).transpose(1, 2).reshape(1, C, H, W)
        elif st == wl.FFN:
            xt = x.flatten(2).transpose(1, 2)
            h = xt @ t(p["w1"]) + t(p["b1"])
            a, g = h.chunk(2, dim=-1)
            x = (xt + (a * F.gelu(g)) @ t(p["w2"]) + t(p["b2"])).transpose(1, 2).reshape(1, C, H, W)
        elif st in (wl.ASATTN, wl.AMLP):
            xt = x.flatten(2).transpose(1, 2)
            sh, sc, g = F.linear(F.silu(t(temb)), t(p["wm"]).T, t(p["bm"])).chunk(3)
            u = F.layer_norm(xt, (C,), None, None, cfg.eps) * (1 + sc) + sh
            if st == wl.ASATTN:
                d = mha(u @ t(p["wq"]), u @ t(p["wk"]), u @ t(p["wv"])) @ t(p["wo"]) + t(p["bo"])
            else:
                d = F.gelu(u @ t(p["w1"]) + t(p["b1"]), approximate="tanh") @ t(p["w2"]) + t(p["b2"])
            x = (xt + g * d).transpose(1, 2).reshape(1, C, H, W)
        elif st in (wl.LSATTN, wl.LXATTN, wl.LFFN):
            xt = x.flatten(2).transpose(1, 2)
            u = F.layer_norm(xt, (C,), t(p["ln_g"]), t(p["ln_b"]), cfg.eps)
            if st == wl.LSATTN:
                d = mha(u @ t(p["wq"]), u @ t(p["wk"]), u @ t(p["wv"])) @ t(p["wo"]) + t(p["bo"])
            elif st == wl.LXATTN:
                c = t(ctx)[None]
                d = mha(u @ t(p["wq"]), c @ t(p["wk"]), c @ t(p["wv"])) @ t(p["wo"]) + t(p["bo"])
            else:
                a, g = (u @ t(p["w1"]) + t(p["b1"])).chunk(2, dim=-1)
                d = (a * F.gelu(g)) @ t(p["w2"]) + t(p["b2"])
            x = (xt + d).transpose(1, 2).reshape(1, C, H, W)
    return x[0].numpy()


@pytest.mark.parametrize("stages", [
    (wl.RES1, wl.SATTN), (wl.RES2,), (wl.SATTN, wl.XATTN, wl.FFN), (wl.RES2, wl.SATTN, wl.XATTN),
    (wl.LSATTN, wl.LXATTN, wl.LFFN), (wl.RES2, wl.LSATTN, wl.LFFN), (wl.RES2T, wl.LSATTN),
    (wl.ASATTN, wl.AMLP)])
def test_block_vs_torch_composition(stages):
    cfg = wl.custom_config([(6, 8), (4, 4)], (2, 2), C=16, G=4, heads=2, stages=stages,
                           ctx_len=5, ctx_dim=12, seed=99, temb_dim=10)
    w = wl.make_workload(cfg)
    for i, z in enumerate(w.images):
        y, _ = ob.block_forward(z, cfg.stages, w.params, G=cfg.G, heads=cfg.heads, eps=cfg.eps, ctx=w.ctx[i],
                                temb=w.temb[i])
        ref = _torch_block(z, cfg, w.params, w.ctx[i], w.temb[i])
        assert np.allclose(y, ref, atol=1e-10), np.abs(y - ref).max()


def test_block_rows_subset_matches_full():
    cfg = wl.custom_config([(6, 8)], (2, 2), C=16, G=4, heads=2, stages=(wl.RES2, wl.SATTN, wl.XATTN, wl.FFN),
                           ctx_len=5, ctx_dim=12, seed=5)
    w = wl.make_workload(cfg)
    full, _ = ob.block_forward(w.images[0], cfg.stages, w.params, G=cfg.G, heads=cfg.heads, ctx=w.ctx[0])
    rows = np.array([3, 47, 20, 0])
    sub, _ = ob.block_forward(w.images[0], cfg.stages, w.params, G=cfg.G, heads=cfg.heads, ctx=w.ctx[0], rows=rows)
    assert np.allclose(sub, full.reshape(16, -1).T[rows], atol=1e-12)


@pytest.mark.parametrize("stages", [(wl.RES2, wl.SATTN), (wl.SATTN,), (wl.RES2, wl.LSATTN, wl.LFFN)])
def test_block_rows_subset_with_reuse_matches_full(stages):
    """Sampled query rows under a reuse mask: the rows that fall on reused patches are the cached output, the others
    the fresh one, and every operand slot after the call is the one of the full run (the exit used for the large image
    of the skewed configuration)."""
    cfg = wl.custom_config([(8, 12)], (4, 4), C=16, G=4, heads=2, stages=stages, reuse_p=0.5, seed=17)
    w = wl.make_workload(cfg)
    c0 = {k: v[0] for k, v in w.cache.items()}
    assert w.reuse[0].any() and not w.reuse[0].all()
    full, nc_full = ob.block_forward(w.images[0], cfg.stages, w.params, G=cfg.G, heads=cfg.heads, reuse=w.reuse[0], cache=c0)
    rows = np.arange(0, 96, 5)                                   # rows on reused and on computed patches
    px = np.kron(w.reuse[0], np.ones((4, 4))).astype(bool).reshape(-1)
    assert px[rows].any() and not px[rows].all()
    sub, nc_sub = ob.block_forward(w.images[0], cfg.stages, w.params, G=cfg.G, heads=cfg.heads, reuse=w.reuse[0], cache=c0,
                                   rows=rows)
    assert np.allclose(sub, full.reshape(16, -1).T[rows], atol=1e-12)
    assert np.array_equal(sub[px[rows]], c0["y"].reshape(16, -1).T[rows][px[rows]])
    for name, slot in nc_sub.items():                            # "y" is not formed on a row subset
        assert np.array_equal(slot, nc_full[name]), name
    assert set(nc_full) - set(nc_sub) == {"y"}


# ----------------------------------------------------------------------------- cache reuse semantics
def _reuse_setup():
    cfg = wl.custom_config([(8, 8), (4, 8)], (4, 4), C=8, G=2, heads=2, stages=(wl.RES2, wl.SATTN),
                           reuse_p=0.5, seed=3)
    return cfg, wl.make_workload(cfg)


def test_reuse_none_equals_ordinary_and_refreshes_every_slot():
    cfg, w = _reuse_setup()
    none = [np.zeros_like(m) for m in w.reuse]
    y0, _ = ob.forward_batch(w.images, cfg.stages, w.params, G=cfg.G, heads=cfg.heads)
    y1, nc = ob.forward_batch(w.images, cfg.stages, w.params, G=cfg.G, heads=cfg.heads, reuse=none, cache=w.cache)
    for a, b, c, z in zip(y0, y1, nc, w.images):
        assert np.array_equal(a, b)
        assert np.array_equal(c["y"], a)
        # slot "1.r" is then the plain RES2 output
        r, _ = ob.block_forward(z, (wl.RES2,), w.params[:1], G=cfg.G, heads=cfg.heads)
        assert np.allclose(c["1.r"], r, atol=1e-13)


def test_reuse_all_returns_cache_and_keeps_slots():
    cfg, w = _reuse_setup()
    allm = [np.ones_like(m) for m in w.reuse]
    y, nc = ob.forward_batch(w.images, cfg.stages, w.params, G=cfg.G, heads=cfg.heads, reuse=allm, cache=w.cache)
    for i in range(cfg.n):
        assert np.array_equal(y[i], w.cache["y"][i].astype(np.float64))
        for k in w.cache:
            assert np.array_equal(nc[i][k], w.cache[k][i].astype(np.float64))


def test_reuse_mixed_follows_operand_fill_rule():
    """Recompute the mixed case with torch pieces, filling operands by hand at each context boundary."""
    cfg, w = _reuse_setup()
    y, nc = ob.forward_batch(w.images, cfg.stages, w.params, G=cfg.G, heads=cfg.heads, reuse=w.reuse, cache=w.cache)
    ph, pw = cfg.patch
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    for i, z in enumerate(w.images):
        m = t(np.kron(w.reuse[i].astype(np.float64), np.ones((ph, pw)))).bool()[None, None]
        C, H, W = z.shape
        p0, p1 = w.params
        x = t(z)[None]
        h1 = F.conv2d(F.silu(F.group_norm(x, cfg.G, t(p0["gn_a_g"]), t(p0["gn_a_b"]), cfg.eps)),
                      t(p0["conv_a_w"]), t(p0["conv_a_b"]), padding=1)
        h1 = torch.where(m, t(w.cache["0.h1"][i])[None], h1)
        r = x + F.conv2d(F.silu(F.group_norm(h1, cfg.G, t(p0["gn_b_g"]), t(p0["gn_b_b"]), cfg.eps)),
                         t(p0["conv_b_w"]), t(p0["conv_b_b"]), padding=1)
        r = torch.where(m, t(w.cache["1.r"][i])[None], r)
        u = F.group_norm(r, cfg.G, t(p1["gn_g"]), t(p1["gn_b"]), cfg.eps).flatten(2).transpose(1, 2)
        mt = m.flatten(2).transpose(1, 2)
        q = u @ t(p1["wq"])
        k = torch.where(mt, t(w.cache["1.K"][i]).flatten(1).T[None], u @ t(p1["wk"]))
        v = torch.where(mt, t(w.cache["1.V"][i]).flatten(1).T[None], u @ t(p1["wv"]))
        hd = cfg.heads
        sp = lambda a: a.reshape(1, -1, hd, C // hd).transpose(1, 2)
        o = F.scaled_dot_product_attention(sp(q), sp(k), sp(v)).transpose(1, 2).reshape(1, -1, C)
        out = r + (o @ t(p1["wo"]) + t(p1["bo"])).transpose(1, 2).reshape(1, C, H, W)
        out = torch.where(m, t(w.cache["y"][i])[None], out)
        assert np.allclose(y[i], out[0].numpy(), atol=1e-10)
        assert np.allclose(nc[i]["0.h1"], h1[0].numpy(), atol=1e-10)
        assert np.allclose(nc[i]["1.K"], k[0].T.reshape(C, H, W).numpy(), atol=1e-10)
        # reused regions of the output are the cache bit for bit
        mm = m[0, 0].numpy()
        assert np.array_equal(y[i][:, mm], w.cache["y"][i].astype(np.float64)[:, mm])


def test_batch_independence():
    cfg, w = _reuse_setup()
    y_all, _ = ob.forward_batch(w.images, cfg.stages, w.params, G=cfg.G, heads=cfg.heads)
    y_one, _ = ob.forward_batch(w.images[1:], cfg.stages, w.params, G=cfg.G, heads=cfg.heads)
    assert np.array_equal(y_all[1], y_one[0])


# ----------------------------------------------------------------------------- planner tables
def _read_golden(path):
    tabs = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *v = line.split()
            v = [int(a) for a in v]
            if k in ("neighbour", "halo_src"):
                tabs.setdefault(k, {})[v[0]] = v[1:]
            else:
                tabs[k] = v
    for k in ("neighbour", "halo_src"):
        tabs[k] = [tabs[k][i] for i in range(len(tabs[k]))]
    return tabs


def test_plan_tables_vs_hand_derived_example():
    g = _read_golden(os.path.join(os.path.dirname(__file__), "golden", "plan_tiny.txt"))
    t = op.plan_tables([(4, 4), (2, 2)], 2, 2)
    for k, v in g.items():
        assert np.array_equal(np.asarray(t[k]).reshape(-1), np.asarray(v).reshape(-1)), k


def test_plan_patch_counts_of_the_benchmark_configs():
    # 4+9 = 13, 4+9+16 = 29, 64+64 = 128 patches
    assert op.plan_tables([(16, 16), (24, 24)], 8, 8)["P"] == 13
    assert op.plan_tables([(64, 64), (96, 96), (128, 128)], 32, 32)["P"] == 29
    assert op.plan_tables([(256, 256)] + [(64, 64)] * 16, 32, 32)["P"] == 128


def test_plan_gcd_patch_and_csp_range_property():
    res = [(96, 64), (32, 32), (64, 96), (32, 32), (64, 96)]
    t = op.plan_tables(res)                      # (0, 0): patch = gcd per dimension
    assert (t["ph"], t["pw"]) == (32, 32)
    ro, own, perm = t["request_offset"], t["patch_owner"], t["perm"]
    # requests sorted by resolution, stable in arrival order
    assert [res[i] for i in perm] == sorted(res)
    assert list(perm) == [1, 3, 2, 4, 0]
    # patches of slot s are exactly RequestOffset[s] .. RequestOffset[s+1]
    for s in range(len(res)):
        H, W = res[perm[s]]
        assert ro[s + 1] - ro[s] == (H // 32) * (W // 32)
        assert (own[ro[s]:ro[s + 1]] == s).all()
    # resolution offsets delimit slots of equal resolution
    for k in range(len(t["res_hw"])):
        for s in range(t["res_offset"][k], t["res_offset"][k + 1]):
            assert tuple(t["res_hw"][k]) == res[perm[s]]
    # neighbour relation is symmetric with mirrored direction; never crosses images
    nb = t["neighbour"]
    for p in range(t["P"]):
        for k in range(8):
            q = nb[p, k]
            if q >= 0:
                assert own[q] == own[p] and nb[q, 7 - k] == p


def test_split_reassemble_vs_einops_and_roundtrip():
    import einops
    imgs = [RNG.standard_normal((3, 4, 6)).astype(np.float32), RNG.standard_normal((3, 2, 2)).astype(np.float32)]
    x = op.split(imgs, 2, 2)
    # sorted order: the 2x2 image first
    e1 = einops.rearrange(imgs[1], "c (r y) (k x) -> (r k y x) c", y=2, x=2)
    e0 = einops.rearrange(imgs[0], "c (r y) (k x) -> (r k y x) c", y=2, x=2)
    assert np.array_equal(x, np.concatenate([e1, e0]))
    back = op.reassemble(x, [(4, 6), (2, 2)], 2, 2)
    assert all(np.array_equal(a, b) for a, b in zip(back, imgs))
    # halo table agrees with split: ring token ids address the right pixels
    t = op.plan_tables([(4, 6), (2, 2)], 2, 2)
    big = imgs[0]
    for p in range(1, t["P"]):
        r, c = t["patch_rc"][p]
        ring = [(-1, xx) for xx in range(-1, 3)] + [(2, xx) for xx in range(-1, 3)] + [(yy, -1) for yy in range(2)] \
            + [(yy, 2) for yy in range(2)]
        for k, (yy, xx) in enumerate(ring):
            Y, X = r * 2 + yy, c * 2 + xx
            tok = t["halo_src"][p, k]
            if 0 <= Y < 4 and 0 <= X < 6:
                assert np.array_equal(x[tok], big[:, Y, X])
            else:
                assert tok == -1


# ----------------------------------------------------------------------------- input generator
def test_generator_is_deterministic_and_standard_normal():
    a = wl.Stream(1, "a").normal((1000, 100))
    b = wl.Stream(1, "a").normal((1000, 100))
    c = wl.Stream(1, "b").normal((1000, 100))
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    assert abs(a.mean()) < 0.01 and abs(a.std() - 1) < 0.01
    # chunked generation equals one-shot generation
    assert np.array_equal(wl.Stream(1, "a").normal((1000, 100), chunk=777), a)
    # known SplitMix64 outputs for seed 0 (reference values of the published generator)
    s = wl.Stream.__new__(wl.Stream)
    s._seed, s._pos = 0, 0
    assert [int(v) for v in s.raw(3)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_bf16_rounding_ties_to_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 3.14159], dtype=np.float32)
    # 1 + 2^-8 is a tie between 1 and 1+2^-7 -> even mantissa (1.0); 1 + 3*2^-8 ties -> 1+2^-6
    r = wl.bf16_round(x)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == np.float32(1.015625) and r[3] == -1.0
    assert np.array_equal(r, torch.from_numpy(x).to(torch.bfloat16).float().numpy())
    assert np.array_equal(wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(r)), r)


def test_config_shapes():
    assert wl.config(1).P == 13 and wl.config(2).P == 29 and wl.config(5).P == 128
    assert wl.config(2).T == 29696 and wl.config(5).T == 131072
    c3, c4 = wl.config(3), wl.config(4)
    assert c3.n == 8 and c4.n == 24 and 32 <= c3.P <= 128 and 96 <= c4.P <= 384


# ----------------------------------------------------------------------------- cache manager pieces
def _mse_images(seed, res, C):
    return [wl.Stream(seed, f"m{i}").normal((C, h, w)).astype(np.float64) for i, (h, w) in enumerate(res)]


def test_patch_mse_closed_forms_and_patch_localisation():
    """Section "Patch-aware Caching Strategy", step 1 (input compared with the cache per patch; metric MSE)."""
    res, ph, pw, C = [(8, 4), (4, 4), (8, 8)], 4, 2, 3
    a = _mse_images(3, res, C)
    assert np.array_equal(oc.patch_mse(a, a, ph, pw), np.zeros(2 * 2 + 1 * 2 + 2 * 4))          # identical -> 0
    b = [x + 0.5 for x in a]
    assert np.allclose(oc.patch_mse(a, b, ph, pw), 0.25, rtol=0, atol=1e-15)                      # constant offset c -> c^2
    # one element changed by d: exactly one patch is non-zero, d^2 / (ph*pw*C), and it is the patch that the
    # (independently pinned) planner tables place at that pixel
    tabs = op.plan_tables(res, ph, pw)
    for img, ch, Y, X in [(0, 1, 5, 3), (2, 0, 7, 0), (1, 2, 0, 3)]:
        b = [x.copy() for x in a]
        b[img][ch, Y, X] += 3.0
        got = oc.patch_mse(a, b, ph, pw)
        slot = list(tabs["perm"]).index(img)
        want = [p for p in range(len(got)) if tabs["patch_owner"][p] == slot
                and tuple(tabs["patch_rc"].reshape(-1, 2)[p]) == (Y // ph, X // pw)]
        assert len(want) == 1
        assert np.flatnonzero(got).tolist() == want
        assert abs(got[want[0]] - 9.0 / (ph * pw * C)) < 1e-15


def test_patch_mse_vs_plain_loops():
    res, ph, pw, C = [(4, 6), (2, 2)], 2, 2, 2
    a, b = _mse_images(5, res, C), _mse_images(6, res, C)
    got = oc.patch_mse(a, b, ph, pw)
    order = sorted(range(len(res)), key=lambda i: (res[i], i))
    k = 0
    for i in order:
        for r in range(res[i][0] // ph):
            for c in range(res[i][1] // pw):
                acc = 0.0
                for ch in range(C):
                    for y in range(ph):
                        for x in range(pw):
                            d = float(a[i][ch, r * ph + y, c * pw + x]) - float(b[i][ch, r * ph + y, c * pw + x])
                            acc += d * d
                assert abs(got[k] - acc / (ph * pw * C)) < 1e-12
                k += 1
    assert k == len(got)


def _read_sets_golden():
    out = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "cache_sets_tiny.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *vals = line.split()
        out[key] = [int(v) for v in vals]
    return out


def test_cache_sets_vs_hand_derived_example():
    """Section "Batching Patches in Cache": Common / New / Expired sets."""
    g = _read_sets_golden()
    old_res = list(zip(g["old_res"][0::2], g["old_res"][1::2]))
    new_res = list(zip(g["new_res"][0::2], g["new_res"][1::2]))
    got = oc.cache_sets(old_res, g["old_ids"], new_res, g["new_ids"], 2, 2)
    assert got["req_src"].tolist() == g["req_src"]
    assert got["expired"].tolist() == g["expired"]
    assert got["patch_src"].tolist() == g["patch_src"]


def test_cache_sets_invariants():
    rng = np.random.default_rng(1)
    sizes = [(4, 4), (8, 4), (8, 8)]
    old_ids = [int(v) for v in rng.permutation(40)[:9]]
    old_res = [sizes[int(rng.integers(3))] for _ in old_ids]
    keep = [i for i in range(9) if rng.random() < 0.6]
    new_ids = [old_ids[i] for i in keep] + [100, 101, 102]
    new_res = [old_res[i] for i in keep] + [sizes[0], sizes[2], sizes[1]]
    order = rng.permutation(len(new_ids))
    new_ids = [new_ids[i] for i in order]
    new_res = [new_res[i] for i in order]
    got = oc.cache_sets(old_res, old_ids, new_res, new_ids, 4, 4)
    # same batch twice: everything is common and the patch table is the identity
    same = oc.cache_sets(old_res, old_ids, old_res, old_ids, 4, 4)
    assert same["patch_src"].tolist() == list(range(len(same["patch_src"]))) and not same["expired"].any()
    # counts: common requests = kept ones; sources are distinct old patches; expired = not kept
    assert int((got["req_src"] >= 0).sum()) == len(keep)
    src = got["patch_src"][got["patch_src"] >= 0]
    assert len(set(src.tolist())) == len(src)
    assert got["expired"].tolist() == [0 if i in keep else 1 for i in range(9)]
    # a migrated slot holds, for a common patch, the old patch's rows
    S, C = 16, 2
    old_slot = rng.standard_normal((len(same["patch_src"]) * S, C))
    fill = np.zeros((len(got["patch_src"]) * S, C))
    new_slot = oc.migrate(old_slot, got["patch_src"], S, fill)
    for p, q in enumerate(got["patch_src"]):
        want = old_slot[q * S:(q + 1) * S] if q >= 0 else 0.0
        assert np.array_equal(new_slot[p * S:(p + 1) * S], want + np.zeros((S, C)))


# ----------------------------------------------------------------------------- resolution changes
def _rs_inputs(C=5, Co=3, H=6, W=8, seed=31):
    u = wl.Stream(seed, "u").normal((C, H, W)).astype(np.float64)
    k = wl.Stream(seed, "k").normal((Co, C, 3, 3)).astype(np.float64)
    b = wl.Stream(seed, "b").normal((Co,)).astype(np.float64)
    return u, k, b


def test_down2_up2_vs_torch_library():
    u, k, b = _rs_inputs()
    t = torch.from_numpy
    ref = F.conv2d(t(u)[None], t(k), t(b), stride=2, padding=1)[0].numpy()
    assert np.allclose(orr.down2(u, k, b), ref, atol=1e-12)
    ref = F.conv2d(F.interpolate(t(u)[None], scale_factor=2, mode="nearest"), t(k), t(b), padding=1)[0].numpy()
    assert np.allclose(orr.up2(u, k, b), ref, atol=1e-12)


def test_down2_closed_forms_fix_centre_stride_and_padding():
    """Centre tap alone: plain subsampling of the even pixels; tap (0, 0) alone: pixel (2oy-1, 2ox-1), zero in the
    first output row and column; all-ones kernel on an all-ones image: the number of taps inside the image."""
    u, _, _ = _rs_inputs(C=2, Co=2)
    eye = np.zeros((2, 2, 3, 3))
    eye[0, 0, 1, 1] = eye[1, 1, 1, 1] = 1.0
    assert np.array_equal(orr.down2(u, eye, np.zeros(2)), u[:, ::2, ::2])
    k00 = np.zeros((2, 2, 3, 3))
    k00[0, 1, 0, 0] = 1.0                                          # out channel 0 reads in channel 1
    y = orr.down2(u, k00, np.zeros(2))
    assert np.array_equal(y[0, 1:, 1:], u[1, 1:-1:2, 1:-1:2]) and not y[0, 0].any() and not y[0, :, 0].any() and not y[1].any()
    ones = orr.down2(np.ones((1, 6, 8)), np.ones((1, 1, 3, 3)), np.array([0.5]))
    want = np.full((3, 4), 9.0)
    want[0, :] = 6.0
    want[:, 0] = 6.0
    want[0, 0] = 4.0                                               # only the top / left border loses taps (even sizes)
    assert np.array_equal(ones[0], want + 0.5)


def test_up2_closed_forms_and_plain_loops():
    """Centre tap alone: every pixel repeated 2 x 2; and a 7-loop evaluation of the definition on a tiny case."""
    u, k, b = _rs_inputs(C=2, Co=2, H=3, W=4)
    eye = np.zeros((2, 2, 3, 3))
    eye[0, 0, 1, 1] = eye[1, 1, 1, 1] = 1.0
    assert np.array_equal(orr.up2(u, eye, np.zeros(2)), np.kron(u, np.ones((2, 2))))
    got = orr.up2(u, k, b)
    for co in range(2):
        for oy in range(6):
            for ox in range(8):
                acc = b[co]
                for ci in range(2):
                    for ty in range(3):
                        for tx in range(3):
                            Y, X = oy + ty - 1, ox + tx - 1
                            if 0 <= Y < 6 and 0 <= X < 8:
                                acc += k[co, ci, ty, tx] * u[ci, Y // 2, X // 2]
                assert abs(got[co, oy, ox] - acc) < 1e-12
    got = orr.down2(u[:, :2, :], k, b)
    for co in range(2):
        for oy in range(1):
            for ox in range(2):
                acc = b[co]
                for ci in range(2):
                    for ty in range(3):
                        for tx in range(3):
                            Y, X = 2 * oy + ty - 1, 2 * ox + tx - 1
                            if 0 <= Y < 2 and 0 <= X < 4:
                                acc += k[co, ci, ty, tx] * u[ci, Y, X]
                assert abs(got[co, oy, ox] - acc) < 1e-12


# ----------------------------------------------------------------------------- scheduler pieces
def _T(i, hw, steps, arrival, ddl, sa):
    return osc.Task(i, hw, hw, steps, float(arrival), float(ddl), float(sa))


def test_slack_and_latency_model_by_hand():
    """Slack = (DDL - C - P) / SA with the numbers of the section's definition worked by hand; the model's features
    for a 64x64 + 64x64 + 128x128 batch at 32x32 patches are 4 + 4 + 16 patches, 2 resolutions and
    1e-6 (4096^2 + 4096^2 + 16384^2) = 301.989888."""
    t = _T(1, 64, 10, 50, 200, 20)
    assert osc.slack(t, 100.0, 3.5) == (200.0 - 50.0 - 35.0) / 20.0 == 5.75
    assert not osc.time_out(t, 100.0, 3.5) and osc.time_out(t, 100.0, 15.1)         # 100 + 151 > 250
    batch = [_T(1, 64, 1, 0, 1, 1), _T(2, 64, 1, 0, 1, 1), _T(3, 128, 1, 0, 1, 1)]
    assert osc.features(batch, 32, 32) == (24.0, 2.0, 301.989888)
    assert abs(osc.predict([2.0, 0.5, 3.0, 0.01], batch, 32, 32) - (2.0 + 12.0 + 6.0 + 3.01989888)) < 1e-12


def test_latency_fit_recovers_a_linear_law():
    rng = np.random.default_rng(5)
    X = rng.uniform(1, 50, size=(40, 3))
    w = np.array([1.5, 0.25, 2.0, 0.125])
    y = w[0] + X @ w[1:]
    assert np.allclose(osc.fit(X, y), w, atol=1e-9)


def test_schedule_hand_derived_scenarios():
    """Latency law 1 + 0.5 * patches (32x32 patches: 32^2 = 1, 64^2 = 4, 128^2 = 16 patches), now = 100.

    A. active {64^2, 10 steps, arrival 0, DDL 300, SA 50}; waiting W0 {32^2, 10 steps, arr 50, DDL 200, SA 20},
       W1 {128^2, 40 steps, arr 0, DDL 500, SA 200}, W2 {64^2, 5 steps, arr 90, DDL 100, SA 50}; relaxed slack 2.
       Slacks in the batch each would join: W0 (200-50-35)/20 = 5.75, W1 (500-100-440)/200 = -0.2, W2 (100-10-25)/50 = 1.3.
       W1 first: 100 + 40*11 = 540 > 500, discarded.  W2 next (1.3 <= 2: urgent mode): the active task ends at
       100 + 10*5 = 150 <= 300, admitted.  W0 last (slack (200-50-55)/20 = 4.75 > 2: throughput mode, sole candidate);
       most urgent active is W2 (1.3 against 3.0), 100 + 5*5.5 = 127.5 <= 190, admitted.  -> admitted [2, 0], discarded [1]
    B. active {64^2, 20 steps, arr 0, DDL 165, SA 50} (alone: ends at 160); waiting {32^2, 2 steps}: with it the
       active task would end at 100 + 20*3.5 = 170 > 165 -> stop, nothing admitted.
    C. nothing active; waiting W0 {64^2, SA 50} slack (1000-100-30)/50 = 17.4, W1 {128^2, SA 10} slack
       (1000-100-90)/10 = 81: least slack is W0 but 17.4 > 2, throughput mode: 4096/3 = 1365 against 16384/9 = 1820
       tokens per ms -> W1 first, then W0.  -> admitted [1, 0]"""
    w = [1.0, 0.5, 0.0, 0.0]
    act = [_T(9, 64, 10, 0, 300, 50)]
    wait = [_T(0, 32, 10, 50, 200, 20), _T(1, 128, 40, 0, 500, 200), _T(2, 64, 5, 90, 100, 50)]
    assert osc.schedule(wait, act, 100.0, w, 32, 32, 2.0) == ([2, 0], [1])
    act = [_T(9, 64, 20, 0, 165, 50)]
    wait = [_T(0, 32, 2, 95, 100, 10)]
    assert osc.schedule(wait, act, 100.0, w, 32, 32, 100.0) == ([], [])
    wait = [_T(0, 64, 10, 0, 1000, 50), _T(1, 128, 10, 0, 1000, 10)]
    assert osc.schedule(wait, [], 100.0, w, 32, 32, 2.0) == ([1, 0], [])
    assert osc.schedule(wait, [], 100.0, w, 32, 32, 50.0) == ([0, 1], [])            # urgent mode: slack order


# ----------------------------------------------------------------------------- joint text-image block
def _mmdit_params(seed, C, D, F):
    rd = lambda name, shape, scale: (wl.Stream(seed, name).normal(shape) * scale).astype(np.float64)
    p = {}
    for X in ("img", "txt"):
        p[X + ".wm"], p[X + ".bm"] = rd(X + "wm", (D, 6 * C), D ** -0.5), rd(X + "bm", (6 * C,), 0.1)
        for n in ("wq", "wk", "wv", "wo"):
            p[X + "." + n] = rd(X + n, (C, C), C ** -0.5)
        p[X + ".bo"] = rd(X + "bo", (C,), 0.1)
        p[X + ".w1"], p[X + ".b1"] = rd(X + "w1", (C, F), C ** -0.5), rd(X + "b1", (F,), 0.1)
        p[X + ".w2"], p[X + ".b2"] = rd(X + "w2", (F, C), F ** -0.5), rd(X + "b2", (C,), 0.1)
    return p


def test_mmdit_vs_torch_composition():
    C, D, Fh, L, heads = 16, 10, 32, 7, 2
    p = _mmdit_params(3, C, D, Fh)
    z = wl.Stream(3, "z").normal((C, 4, 6)).astype(np.float64)
    txt = wl.Stream(3, "t").normal((L, C)).astype(np.float64)
    c = wl.Stream(3, "c").normal((D,)).astype(np.float64)
    gi, gt = ob.mmdit(z, txt, c, p, heads, 1e-5)
    t = torch.from_numpy
    xs = {"img": t(z).flatten(1).T, "txt": t(txt)}
    mod, qkv = {}, {}
    for X in ("img", "txt"):
        mod[X] = F_linear(F.silu(t(c)), t(p[X + ".wm"]), t(p[X + ".bm"])).chunk(6)
        h = F.layer_norm(xs[X], (C,), None, None, 1e-5) * (1 + mod[X][1]) + mod[X][0]
        qkv[X] = [h @ t(p[X + "." + n]) for n in ("wq", "wk", "wv")]
    cat = [torch.cat([qkv["img"][i], qkv["txt"][i]]) for i in range(3)]
    sp = lambda a: a.reshape(1, -1, heads, C // heads).transpose(1, 2)
    o = F.scaled_dot_product_attention(sp(cat[0]), sp(cat[1]), sp(cat[2])).transpose(1, 2).reshape(-1, C)
    outs, at = {}, 0
    for X in ("img", "txt"):
        n = xs[X].shape[0]
        x1 = xs[X] + mod[X][2] * (o[at:at + n] @ t(p[X + ".wo"]) + t(p[X + ".bo"]))
        at += n
        h2 = F.layer_norm(x1, (C,), None, None, 1e-5) * (1 + mod[X][4]) + mod[X][3]
        outs[X] = x1 + mod[X][5] * (F.gelu(h2 @ t(p[X + ".w1"]) + t(p[X + ".b1"]), approximate="tanh") @ t(p[X + ".w2"]) + t(p[X + ".b2"]))
    assert np.allclose(gi, outs["img"].T.reshape(C, 4, 6).numpy(), atol=1e-10)
    assert np.allclose(gt, outs["txt"].numpy(), atol=1e-10)


def F_linear(x, w, b):
    return x @ w + b


def test_mmdit_without_text_is_the_adaln_block_and_text_order_is_free():
    """No text tokens: the image stream is ASATTN followed by AMLP with the modulation split in two (both pinned
    above).  With text: permuting the text tokens permutes the text output and leaves the image output alone."""
    C, D, Fh, heads = 16, 10, 32, 2
    p = _mmdit_params(4, C, D, Fh)
    z = wl.Stream(4, "z").normal((C, 4, 6)).astype(np.float64)
    c = wl.Stream(4, "c").normal((D,)).astype(np.float64)
    gi, gt = ob.mmdit(z, np.zeros((0, C)), c, p, heads, 1e-5)
    assert gt.shape == (0, C)
    pa = {"wm": p["img.wm"][:, :3 * C], "bm": p["img.bm"][:3 * C], **{n: p["img." + n] for n in ("wq", "wk", "wv", "wo", "bo")}}
    pm = {"wm": p["img.wm"][:, 3 * C:], "bm": p["img.bm"][3 * C:], **{n: p["img." + n] for n in ("w1", "b1", "w2", "b2")}}
    ref, _ = ob.block_forward(z, ("ASATTN", "AMLP"), [pa, pm], G=1, heads=heads, eps=1e-5, temb=c)
    assert np.allclose(gi, ref, atol=1e-12)
    txt = wl.Stream(4, "t").normal((5, C)).astype(np.float64)
    a_i, a_t = ob.mmdit(z, txt, c, p, heads, 1e-5)
    perm = np.array([3, 0, 4, 1, 2])
    b_i, b_t = ob.mmdit(z, txt[perm], c, p, heads, 1e-5)
    assert np.allclose(a_i, b_i, atol=1e-12) and np.allclose(a_t[perm], b_t, atol=1e-12)
    assert np.abs(a_i - gi).max() > 1e-3                           # the text does reach the image stream


def test_plan_with_text_patches():
    """Text patches sit behind the image patches of their request, off the grid: the image part of every table is the
    plan without text, renumbered; seq_len = H*W + L; the scatter / gather pair round-trips and zero-fills the padding."""
    res, ph, pw, L = [(8, 8), (4, 8), (8, 8)], 4, 4, 20
    a, b = op.plan_tables(res, ph, pw), op.plan_tables(res, ph, pw, text_len=L)
    tp = 2                                                         # ceil(20 / 16)
    assert b["P"] == a["P"] + 3 * tp and b["T"] == b["P"] * 16
    assert np.array_equal(b["perm"], a["perm"]) and np.array_equal(b["seq_len"], [32 + L, 64 + L, 64 + L])
    assert np.array_equal(np.diff(b["request_offset"]), np.diff(a["request_offset"]) + tp)
    img = [q for q in range(b["P"]) if b["patch_rc"][q, 0] >= 0]
    new_id = {old: q for old, q in enumerate(img)}
    assert np.array_equal(b["patch_rc"][img], a["patch_rc"]) and np.array_equal(b["patch_owner"][img], a["patch_owner"])
    remap = lambda v, scale: np.where(v < 0, -1, np.vectorize(lambda u: new_id[u // scale] * scale + u % scale)(np.maximum(v, 0)))
    assert np.array_equal(b["neighbour"][img], remap(a["neighbour"], 1))
    assert np.array_equal(b["halo_src"][img], remap(a["halo_src"], 16))
    txtp = [q for q in range(b["P"]) if b["patch_rc"][q, 0] < 0]
    assert (b["neighbour"][txtp] == -1).all() and (b["halo_src"][txtp] == -1).all()
    assert [tuple(b["patch_rc"][q]) for q in txtp] == [(-1, 0), (-1, 1)] * 3
    x = wl.Stream(9, "x").normal((b["T"], 3))
    text = wl.Stream(9, "t").normal((3, L, 3))
    y = op.text_scatter(x, text, res, ph, pw)
    assert np.array_equal(op.text_gather(y, L, res, ph, pw), text)
    for s in range(3):
        lo, hi = b["cu_seqlens"][s] + b["seq_len"][s], b["cu_seqlens"][s + 1]
        assert hi - lo == tp * 16 - L and not y[lo:hi].any()
        img_rows = slice(b["cu_seqlens"][s], b["cu_seqlens"][s] + b["seq_len"][s] - L)
        assert np.array_equal(y[img_rows], x[img_rows])
