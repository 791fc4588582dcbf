"""CPU oracle of the mixed-resolution denoising block: each image whole and unpatched.

TEST INFRASTRUCTURE ONLY.  This is the slow, plain definition the HIP path is
checked against.  It shares no code with the HIP path, is imported only by the
tests, the smoke check and the CPU-baseline leg of the benchmark, and must never
be used by the product path.

The paper's claim is that running operators on a batch of equal patches of
mixed-resolution images gives the result of running every image on its own
(Patched Inference section; for the convolution-free model the evaluation table
reports PSNR inf / SSIM 1.0 for every patch size).  The method therefore reaches,
up to rounding order, a result with a plain definition, and the oracle is that
definition written out: every function takes ONE image as a float64 array
[C, H, W] and never forms patches, neighbour tables, halos or sequence offsets.
A library matrix product (numpy.matmul) serves as a step; there is no blocking,
fusion or reordering beyond splitting independent query rows into chunks to bound
memory.

Readings of points the paper leaves open (each also listed in the design notes):
  * GroupNorm statistics are taken over the whole image (all its patches), biased
    variance, eps = 1e-5, per-channel affine.
  * "pad with 0 when a neighbour is absent" (Patch-Tailored Diffusion Operators)
    == ordinary zero padding 1 at the true image border.
  * attention: scale 1/sqrt(d), no mask, no positional term (Patch-based
    Self-Attention Module: every query meets all keys of its own image).
  * GELU is the exact erf form; the GEGLU value half comes first, the gate half second.
  * The L-stages (LSATTN, LXATTN, LFFN) are the attention / feed-forward stages with a
    per-pixel LayerNorm over the channels in front (the transformer layer of the
    paper's first model normalises each token before every sub-layer; the paper
    lists such per-pixel operators among those that patching leaves untouched,
    Patch-Tailored Diffusion Operators): biased variance, same eps, per-channel affine.
    Nothing of a reused patch's input is needed by them, so only K and V are cached.
  * ASATTN and AMLP are the self-attention and feed-forward sub-layers of a block of the
    paper's second model family (a diffusion transformer): the request's conditioning
    vector c goes through SiLU and a linear layer to three C-vectors (shift, scale, gate);
    the sub-layer sees LN0(x) * (1 + scale) + shift (LN0: LayerNorm without affine) and
    its output is multiplied by gate before the residual add.  The feed-forward is
    GELU(h W_1 + b_1) W_2 + b_2 with the tanh form of GELU (that model's choice).  The
    joint text-image attention of that model is not part of these stages.
  * MMDIT is a whole joint block of that model (function mmdit): two streams with their own
    weights, one attention over the concatenated image and text tokens of a request.  It is
    called on its own (block_forward carries images only), one request at a time.
  * RES2T is RES2 with the time embedding of the first model's residual block: the
    request's embedding vector goes through SiLU and a linear layer, and the resulting
    C values are added to every pixel of the first convolution's output (a per-pixel
    operator with a per-request operand; the cached h1 of a reused patch includes it).
  * cache reuse (Patch-aware Caching Strategy, steps 3-5): at each operator that
    needs context the operand of a reused patch is the cached tensor of the
    previous step; after the block the reused patches of the output are replaced by
    the cached output; the cache then holds fresh values on computed patches.

Pins (tests/test_oracle_pins.py): 7-loop direct convolution, delta and all-ones
kernels (closed forms fix padding and tap orientation), GroupNorm moments and
shift/scale invariance, three-pass softmax attention, uniform-attention special
case, permutation equivariance, printed constants SiLU(1), GELU(1), and
independent torch CPU library routines.  Absolute block outputs have no value
printed in the paper: "parity unpinned" beyond these pins and the invariants
one-patch == unpatched and patched == per-image.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64


# ----------------------------------------------------------------------------- pointwise
def silu(u: np.ndarray) -> np.ndarray:
    """SiLU(u) = u / (1 + exp(-u))."""
    return u / (1.0 + np.exp(-u))


def gelu_tanh(u: np.ndarray) -> np.ndarray:
    """GELU, tanh form: u/2 * (1 + tanh(sqrt(2/pi) * (u + 0.044715 u^3)))."""
    return 0.5 * u * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (u + 0.044715 * u ** 3)))


def gelu(u: np.ndarray) -> np.ndarray:
    """GELU(u) = u/2 * (1 + erf(u / sqrt 2)) (exact form)."""
    return 0.5 * u * (1.0 + _erf(u / np.sqrt(2.0)))


# ----------------------------------------------------------------------------- GroupNorm
def group_norm(u: np.ndarray, gamma: np.ndarray, beta: np.ndarray, G: int, eps: float) -> np.ndarray:
    """GroupNorm over one whole image u[C, H, W].

    Group g holds channels g*C/G .. (g+1)*C/G-1; mean and biased variance run over
    all H*W*C/G elements of the group (the whole image, not a patch).
    """
    C, H, W = u.shape
    cg = C // G
    out = np.empty_like(u, dtype=F64)
    for g in range(G):
        blk = u[g * cg:(g + 1) * cg].astype(F64)
        mu = blk.mean()
        var = ((blk - mu) ** 2).mean()
        xh = (blk - mu) / np.sqrt(var + eps)
        out[g * cg:(g + 1) * cg] = xh * gamma[g * cg:(g + 1) * cg, None, None] \
            + beta[g * cg:(g + 1) * cg, None, None]
    return out


def layer_norm(u: np.ndarray, gamma: np.ndarray, beta: np.ndarray, eps: float) -> np.ndarray:
    """LayerNorm of every pixel of u[C, H, W] over its C channels (mean and biased variance per pixel)."""
    C, H, W = u.shape
    out = np.empty((C, H, W), dtype=F64)
    for y in range(H):
        for x in range(W):
            v = u[:, y, x].astype(F64)
            mu = v.sum() / C
            var = ((v - mu) ** 2).sum() / C
            out[:, y, x] = (v - mu) / np.sqrt(var + eps) * gamma.astype(F64) + beta.astype(F64)
    return out


# ----------------------------------------------------------------------------- convolution
def conv3(u: np.ndarray, W: np.ndarray, b: np.ndarray) -> np.ndarray:
    """3x3 cross-correlation, stride 1, zero padding 1.

    out[co, y, x] = b[co] + sum_{ci, ky, kx} u[ci, y+ky-1, x+kx-1] * W[co, ci, ky, kx],
    with u taken as 0 outside the image.  One matrix product per tap.
    """
    Ci, H, Wd = u.shape
    Co = W.shape[0]
    up = np.zeros((Ci, H + 2, Wd + 2), dtype=F64)
    up[:, 1:H + 1, 1:Wd + 1] = u
    out = np.zeros((Co, H * Wd), dtype=F64)
    for ky in range(3):
        for kx in range(3):
            window = up[:, ky:ky + H, kx:kx + Wd].reshape(Ci, H * Wd)
            out += W[:, :, ky, kx].astype(F64) @ window
    out += b.astype(F64)[:, None]
    return out.reshape(Co, H, Wd)


# ----------------------------------------------------------------------------- attention
def attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, heads: int,
              rows: Optional[np.ndarray] = None, chunk: int = 1024) -> np.ndarray:
    """Multi-head softmax attention over one token set.

    Q [Nq, C], K [Nk, C], V [Nk, C]; head h uses channel slice h*d .. (h+1)*d-1.
    O_h = softmax_rows(Q_h K_h^T / sqrt(d)) V_h.  `rows` selects query rows (each
    row is independent of the others); query rows are processed in chunks only to
    bound memory.
    """
    if rows is not None:
        Q = Q[rows]
    Nq, C = Q.shape
    d = C // heads
    out = np.empty((Nq, C), dtype=F64)
    for h in range(heads):
        Kh = K[:, h * d:(h + 1) * d].astype(F64)
        Vh = V[:, h * d:(h + 1) * d].astype(F64)
        for r0 in range(0, Nq, chunk):
            Qh = Q[r0:r0 + chunk, h * d:(h + 1) * d].astype(F64)
            S = (Qh @ Kh.T) / np.sqrt(float(d))
            S -= S.max(axis=1, keepdims=True)
            E = np.exp(S)
            A = E / E.sum(axis=1, keepdims=True)
            out[r0:r0 + chunk, h * d:(h + 1) * d] = A @ Vh
    return out


def _tokens(u: np.ndarray) -> np.ndarray:
    """[C, H, W] -> [H*W, C] (token n = y*W + x)."""
    C, H, W = u.shape
    return u.reshape(C, H * W).T


def _image(t: np.ndarray, H: int, W: int) -> np.ndarray:
    return t.T.reshape(t.shape[1], H, W)


def _fill(fresh: np.ndarray, cached: Optional[np.ndarray], reuse_px: Optional[np.ndarray]) -> np.ndarray:
    """Operand-fill rule: cached values on reused pixels, fresh values elsewhere ([C, H, W])."""
    if reuse_px is None:
        return fresh
    return np.where(reuse_px[None, :, :], cached.astype(F64), fresh)


# ----------------------------------------------------------------------------- stages
def res1(x, p, G, eps):
    """RES1(x) = x + conv3(SiLU(GN(x)))."""
    return x + conv3(silu(group_norm(x, p["gn_g"], p["gn_b"], G, eps)), p["conv_w"], p["conv_b"])


def res2(x, p, G, eps, reuse_px=None, cache=None, key="", new_cache=None):
    """RES2(x) = x + conv3_b(SiLU(GN_b(h1))),  h1 = conv3_a(SiLU(GN_a(x))).

    With reuse, h1 of reused patches is the cached h1 (it feeds GN_b statistics and
    the halos of conv_b).
    """
    h1 = conv3(silu(group_norm(x, p["gn_a_g"], p["gn_a_b"], G, eps)), p["conv_a_w"], p["conv_a_b"])
    if reuse_px is not None:
        h1 = _fill(h1, cache[key + "h1"], reuse_px)
        new_cache[key + "h1"] = h1
    return x + conv3(silu(group_norm(h1, p["gn_b_g"], p["gn_b_b"], G, eps)), p["conv_b_w"], p["conv_b_b"])


def res2t(x, p, G, eps, temb, reuse_px=None, cache=None, key="", new_cache=None):
    """RES2T(x) = x + conv3_b(SiLU(GN_b(h1))),  h1 = conv3_a(SiLU(GN_a(x))) + (SiLU(temb) W_t + b_t)[:, None, None].

    temb: the request's embedding vector [D].  With reuse, h1 of reused patches is the cached h1.
    """
    e = silu(np.asarray(temb, dtype=F64)) @ p["wt"].astype(F64) + p["bt"].astype(F64)
    h1 = conv3(silu(group_norm(x, p["gn_a_g"], p["gn_a_b"], G, eps)), p["conv_a_w"], p["conv_a_b"]) + e[:, None, None]
    if reuse_px is not None:
        h1 = _fill(h1, cache[key + "h1"], reuse_px)
        new_cache[key + "h1"] = h1
    return x + conv3(silu(group_norm(h1, p["gn_b_g"], p["gn_b_b"], G, eps)), p["conv_b_w"], p["conv_b_b"])


def sattn(x, p, G, heads, eps, reuse_px=None, cache=None, key="", new_cache=None, rows=None):
    """SATTN(x) = x + concat_h(softmax(Q_h K_h^T / sqrt d) V_h) W_o + b_o, Q/K/V = GN(x) W_{q,k,v}.

    With reuse, the stage input ("r"), K and V of reused patches come from the cache.
    Returns tokens [N or len(rows), C] when rows is given, else an image [C, H, W].
    """
    C, H, W = x.shape
    if reuse_px is not None:
        x = _fill(x, cache[key + "r"], reuse_px)
        new_cache[key + "r"] = x
    u = _tokens(group_norm(x, p["gn_g"], p["gn_b"], G, eps))
    Q = u @ p["wq"].astype(F64)
    K = u @ p["wk"].astype(F64)
    V = u @ p["wv"].astype(F64)
    if reuse_px is not None:
        K = _tokens(_fill(_image(K, H, W), cache[key + "K"], reuse_px))
        V = _tokens(_fill(_image(V, H, W), cache[key + "V"], reuse_px))
        new_cache[key + "K"] = _image(K, H, W)
        new_cache[key + "V"] = _image(V, H, W)
    O = attention(Q, K, V, heads, rows=rows)
    xt = _tokens(x) if rows is None else _tokens(x)[rows]
    yt = xt + O @ p["wo"].astype(F64) + p["bo"].astype(F64)
    return yt if rows is not None else _image(yt, H, W)


def lsattn(x, p, heads, eps, reuse_px=None, cache=None, key="", new_cache=None, rows=None):
    """LSATTN(x) = x + MHA(LN(x)) W_o + b_o.  With reuse, K and V of reused patches come from the cache (the
    normalisation is per pixel, so the stage input of a reused patch is not needed)."""
    C, H, W = x.shape
    u = _tokens(layer_norm(x, p["ln_g"], p["ln_b"], eps))
    Q = u @ p["wq"].astype(F64)
    K = u @ p["wk"].astype(F64)
    V = u @ p["wv"].astype(F64)
    if reuse_px is not None:
        K = _tokens(_fill(_image(K, H, W), cache[key + "K"], reuse_px))
        V = _tokens(_fill(_image(V, H, W), cache[key + "V"], reuse_px))
        new_cache[key + "K"] = _image(K, H, W)
        new_cache[key + "V"] = _image(V, H, W)
    O = attention(Q, K, V, heads, rows=rows)
    xt = _tokens(x) if rows is None else _tokens(x)[rows]
    yt = xt + O @ p["wo"].astype(F64) + p["bo"].astype(F64)
    return yt if rows is not None else _image(yt, H, W)


def _modulation(cvec, p):
    """(shift, scale, gate), each [C]: thirds of SiLU(c) W_m + b_m."""
    m = silu(np.asarray(cvec, dtype=F64)) @ p["wm"].astype(F64) + p["bm"].astype(F64)
    C = m.shape[0] // 3
    return m[:C], m[C:2 * C], m[2 * C:]


def _ln0_mod_tokens(xt, shift, scale, eps):
    """LayerNorm without affine of every row of xt [N, C], then * (1 + scale) + shift."""
    C = xt.shape[1]
    xh = _tokens(layer_norm(_image(xt, xt.shape[0], 1), np.ones(C), np.zeros(C), eps))
    return xh * (1.0 + scale) + shift


def asattn(x, p, heads, eps, cvec, reuse_px=None, cache=None, key="", new_cache=None, rows=None):
    """ASATTN(x) = x + gate * (MHA(h) W_o + b_o), h = LN0(x) * (1 + scale) + shift.  K, V cached like LSATTN."""
    C, H, W = x.shape
    shift, scale, gate = _modulation(cvec, p)
    u = _ln0_mod_tokens(_tokens(x), shift, scale, eps)
    Q = u @ p["wq"].astype(F64)
    K = u @ p["wk"].astype(F64)
    V = u @ p["wv"].astype(F64)
    if reuse_px is not None:
        K = _tokens(_fill(_image(K, H, W), cache[key + "K"], reuse_px))
        V = _tokens(_fill(_image(V, H, W), cache[key + "V"], reuse_px))
        new_cache[key + "K"] = _image(K, H, W)
        new_cache[key + "V"] = _image(V, H, W)
    O = attention(Q, K, V, heads, rows=rows)
    xt = _tokens(x) if rows is None else _tokens(x)[rows]
    yt = xt + gate * (O @ p["wo"].astype(F64) + p["bo"].astype(F64))
    return yt if rows is not None else _image(yt, H, W)


def amlp_tokens(xt, p, eps, cvec):
    """AMLP(x) = x + gate * (GELU_tanh(h W_1 + b_1) W_2 + b_2), h = LN0(x) * (1 + scale) + shift."""
    shift, scale, gate = _modulation(cvec, p)
    h = _ln0_mod_tokens(xt, shift, scale, eps) @ p["w1"].astype(F64) + p["b1"].astype(F64)
    return xt + gate * (gelu_tanh(h) @ p["w2"].astype(F64) + p["b2"].astype(F64))


def _ln_tokens(xt, p, eps):
    """LayerNorm of tokens [N, C] (each row on its own)."""
    return _tokens(layer_norm(_image(xt, xt.shape[0], 1), p["ln_g"], p["ln_b"], eps))


def xattn_tokens(xt, p, heads, ctx):
    """XATTN on tokens [N, C]: queries from x, keys/values from the image's own text tokens."""
    Q = xt @ p["wq"].astype(F64)
    K = ctx.astype(F64) @ p["wk"].astype(F64)
    V = ctx.astype(F64) @ p["wv"].astype(F64)
    O = attention(Q, K, V, heads)
    return xt + O @ p["wo"].astype(F64) + p["bo"].astype(F64)


def ffn_tokens(xt, p):
    """FFN(x) = x + (a * GELU(g)) W_2 + b_2, [a | g] = x W_1 + b_1 (value half first)."""
    h = xt @ p["w1"].astype(F64) + p["b1"].astype(F64)
    F = h.shape[1] // 2
    return xt + (h[:, :F] * gelu(h[:, F:])) @ p["w2"].astype(F64) + p["b2"].astype(F64)


def lxattn_tokens(xt, p, heads, ctx, eps):
    """LXATTN(x) = x + MHA(LN(x) W_q; ctx W_k, ctx W_v) W_o + b_o."""
    Q = _ln_tokens(xt, p, eps) @ p["wq"].astype(F64)
    K = ctx.astype(F64) @ p["wk"].astype(F64)
    V = ctx.astype(F64) @ p["wv"].astype(F64)
    return xt + attention(Q, K, V, heads) @ p["wo"].astype(F64) + p["bo"].astype(F64)


def lffn_tokens(xt, p, eps):
    """LFFN(x) = x + (a * GELU(g)) W_2 + b_2, [a | g] = LN(x) W_1 + b_1."""
    h = _ln_tokens(xt, p, eps) @ p["w1"].astype(F64) + p["b1"].astype(F64)
    F = h.shape[1] // 2
    return xt + (h[:, :F] * gelu(h[:, F:])) @ p["w2"].astype(F64) + p["b2"].astype(F64)


def mmdit(x, txt, cvec, p, heads, eps):
    """One joint block of the paper's second model on ONE request: image x [C, H, W] and its text tokens txt [L, C].

    Each stream X in (img, txt) has its own weights p["X.*"]: six modulation vectors from the request's conditioning
    vector, (sh1, sc1, g1, sh2, sc2, g2) = sixths of SiLU(c) W_m + b_m; q, k, v = h W_q, h W_k, h W_v with
    h = LN0(x) (1 + sc1) + sh1; ONE softmax attention over the concatenated tokens of both streams (every token of the
    request attends to all image and all text tokens of the same request); x += g1 * (o W_o + b_o);
    x += g2 * (GELU_tanh(h2 W_1 + b_1) W_2 + b_2) with h2 = LN0(x) (1 + sc2) + sh2.  Returns (image, text)."""
    C, H, W = x.shape
    streams = {"img": _tokens(np.asarray(x, dtype=F64)), "txt": np.asarray(txt, dtype=F64)}
    mod, q, k, v = {}, {}, {}, {}
    for X, t in streams.items():
        m = silu(np.asarray(cvec, dtype=F64)) @ p[X + ".wm"].astype(F64) + p[X + ".bm"].astype(F64)
        mod[X] = [m[i * C:(i + 1) * C] for i in range(6)]
        h = _ln0_mod_tokens(t, mod[X][0], mod[X][1], eps)
        q[X], k[X], v[X] = (h @ p[X + "." + n].astype(F64) for n in ("wq", "wk", "wv"))
    order = ("img", "txt")
    O = attention(np.concatenate([q[X] for X in order]), np.concatenate([k[X] for X in order]),
                  np.concatenate([v[X] for X in order]), heads)
    out, at = {}, 0
    for X in order:
        t = streams[X]
        o = O[at:at + t.shape[0]]
        at += t.shape[0]
        t = t + mod[X][2] * (o @ p[X + ".wo"].astype(F64) + p[X + ".bo"].astype(F64))
        h2 = _ln0_mod_tokens(t, mod[X][3], mod[X][4], eps)
        t = t + mod[X][5] * (gelu_tanh(h2 @ p[X + ".w1"].astype(F64) + p[X + ".b1"].astype(F64)) @ p[X + ".w2"].astype(F64)
                             + p[X + ".b2"].astype(F64))
        out[X] = t
    return _image(out["img"], H, W), out["txt"]


# ----------------------------------------------------------------------------- whole block
def block_forward(z: np.ndarray, stages: Sequence[str], params: List[Dict[str, np.ndarray]], *,
                  G: int, heads: int, eps: float = 1e-5, ctx: Optional[np.ndarray] = None,
                  reuse: Optional[np.ndarray] = None, cache: Optional[Dict[str, np.ndarray]] = None,
                  rows: Optional[np.ndarray] = None, temb: Optional[np.ndarray] = None):
    """Run the stage list on ONE image z[C, H, W]; returns (out, new_cache).

    reuse: bool [gh, gw] over the image's patch grid (True = reuse the cached
    patch); cache: slot name -> [C, H, W] for this image ("<stage>.h1",
    "<stage>.r", "<stage>.K", "<stage>.V", "y").  new_cache holds every slot after
    the call (fresh on computed patches, unchanged on reused ones).
    rows: optional token subset (n = y*W + x); allowed when every stage from the
    last SATTN on acts per token; then out is [len(rows), C].
    """
    x = np.asarray(z, dtype=F64)
    C, H, W = x.shape
    reuse_px = None
    new_cache: Dict[str, np.ndarray] = {}
    if reuse is not None:
        gh, gw = reuse.shape
        reuse_px = np.repeat(np.repeat(np.asarray(reuse, dtype=bool), H // gh, axis=0), W // gw, axis=1)
    tokens = None                      # set once only sampled rows are carried
    if rows is not None:
        last_ctx = max(i for i, s in enumerate(stages) if s in ("RES1", "RES2", "RES2T", "SATTN", "LSATTN", "ASATTN"))
        assert stages[last_ctx] in ("SATTN", "LSATTN", "ASATTN"), "rows need a self-attention as the last context stage"
    for si, (st, p) in enumerate(zip(stages, params)):
        key = f"{si}."
        if st == "RES1":
            x = res1(x, p, G, eps)
        elif st == "RES2":
            x = res2(x, p, G, eps, reuse_px, cache, key, new_cache)
        elif st == "RES2T":
            x = res2t(x, p, G, eps, temb, reuse_px, cache, key, new_cache)
        elif st == "SATTN":
            if rows is not None and si == last_ctx:
                tokens = sattn(x, p, G, heads, eps, reuse_px, cache, key, new_cache, rows=rows)
            else:
                x = sattn(x, p, G, heads, eps, reuse_px, cache, key, new_cache)
        elif st == "LSATTN":
            if rows is not None and si == last_ctx:
                tokens = lsattn(x, p, heads, eps, reuse_px, cache, key, new_cache, rows=rows)
            else:
                x = lsattn(x, p, heads, eps, reuse_px, cache, key, new_cache)
        elif st == "ASATTN":
            if rows is not None and si == last_ctx:
                tokens = asattn(x, p, heads, eps, temb, reuse_px, cache, key, new_cache, rows=rows)
            else:
                x = asattn(x, p, heads, eps, temb, reuse_px, cache, key, new_cache)
        elif st == "AMLP":
            if tokens is not None:
                tokens = amlp_tokens(tokens, p, eps, temb)
            else:
                x = _image(amlp_tokens(_tokens(x), p, eps, temb), H, W)
        elif st in ("LXATTN", "LFFN"):
            f = (lambda t: lxattn_tokens(t, p, heads, ctx, eps)) if st == "LXATTN" else (lambda t: lffn_tokens(t, p, eps))
            if tokens is not None:
                tokens = f(tokens)
            else:
                x = _image(f(_tokens(x)), H, W)
        elif st == "XATTN":
            if tokens is not None:
                tokens = xattn_tokens(tokens, p, heads, ctx)
            else:
                x = _image(xattn_tokens(_tokens(x), p, heads, ctx), H, W)
        elif st == "FFN":
            if tokens is not None:
                tokens = ffn_tokens(tokens, p)
            else:
                x = _image(ffn_tokens(_tokens(x), p), H, W)
        else:
            raise ValueError(st)
    if tokens is not None:
        if reuse_px is not None:
            ry = _tokens(cache["y"].astype(F64))[rows]
            m = reuse_px.reshape(-1)[rows]
            tokens = np.where(m[:, None], ry, tokens)
        return tokens, new_cache
    if reuse_px is not None:
        x = _fill(x, cache["y"], reuse_px)
        new_cache["y"] = x
    return x, new_cache


def forward_batch(images, stages, params, *, G, heads, eps=1e-5, ctx=None, reuse=None, cache=None, temb=None):
    """Run block_forward on every image of a batch, one at a time (caller order)."""
    outs, caches = [], []
    for i, z in enumerate(images):
        c_i = None if cache is None else {k: v[i] for k, v in cache.items()}
        y, nc = block_forward(z, stages, params, G=G, heads=heads, eps=eps,
                              ctx=None if ctx is None else ctx[i],
                              reuse=None if reuse is None else reuse[i], cache=c_i,
                              temb=None if temb is None else temb[i])
        outs.append(y)
        caches.append(nc)
    return outs, caches
