"""GPU parity on inputs that leave the comfortable range of the seeded N(0,1) workloads.

* attention logits with a wide range, so that the softmax reference of the MFMA kernel has to move after the first
  key tile (the rescale / recompute path), for image keys and for text keys, with both query-tile sizes and a ragged
  last key tile;
* attention logits beyond +-100 (base 2), where the large-tile kernel has to fall back to its second pass;
* GroupNorm inputs whose mean is far from zero (|mean| = 30 standard deviations): the statistics must not lose the
  variance to cancellation.
Bars as everywhere: fp32 within 1e-4 * max|ref|, bf16 within 2e-2 * max|ref|.
"""
import numpy as np
import pytest

import workloads as wl
from oracle import block as ob
from oracle import plan as op
from harness import GpuRun, rel_err, tolerance

pytestmark = pytest.mark.gpu

LOG2E = 1.4426950408889634


def _oracle(w, reuse=None, cache=None):
    cfg = w.cfg
    return ob.forward_batch(w.images, cfg.stages, w.params, G=cfg.G, heads=cfg.heads, eps=cfg.eps, ctx=w.ctx,
                            reuse=reuse, cache=cache, temb=w.temb)


def _late_maximum_rows(Q, K, heads, first=32, gap=13.0):
    """Number of (head, query) pairs whose largest base-2 logit among the keys behind the first `first` exceeds the
    largest of the first `first` keys by more than `gap`: 2^gap alone is then above any partial-sum threshold up to
    2^12, whatever happened to the reference before."""
    d = Q.shape[1] // heads
    count = 0
    for h in range(heads):
        S2 = (Q[:, h * d:(h + 1) * d] @ K[:, h * d:(h + 1) * d].T) * (LOG2E / np.sqrt(d))
        if S2.shape[1] <= first:
            continue
        count += int((S2[:, first:].max(axis=1) - S2[:, :first].max(axis=1) > gap).sum())
    return count


WIDE = [
    # few query tiles: the launch takes the small query tile; 144 = 2 * 64 + 16 keys (ragged last key tile)
    ("few", [(16, 16), (24, 16), (12, 12)]),
    # many query tiles (>= 1,024 with two heads): the large query tile; 144 and 400 = 6 * 64 + 16 keys
    ("many", [(12, 12)] * 384 + [(20, 20)] * 128),
]


@pytest.mark.parametrize("stage", [wl.SATTN, wl.XATTN])
@pytest.mark.parametrize("name,res", WIDE, ids=[c[0] for c in WIDE])
def test_attention_wide_logits(name, res, stage):
    """Self- and cross-attention (head dim 64, bf16) whose softmax reference must move after the first key tile: the
    first 32 keys of every request (its first two 4 x 4 patches, resp. its first 32 text tokens) are damped to 5 % and
    the query projection is scaled by 4, so that the logits of the later keys span tens of units while the first 32
    stay near zero.  (A larger scale would test bf16 rounding of the logits rather than the kernel: the error of an
    exact softmax on bf16-rounded q and k already reaches 1.6e-2 at scale 8.)"""
    cfg = wl.custom_config(res, (4, 4), C=128, G=32, heads=2, stages=(stage,), dtype="bf16", ctx_len=77, ctx_dim=64, seed=77)
    w = wl.make_workload(cfg)
    p = w.params[0]
    p["wq"] = p["wq"] * np.float32(4.0)                          # a power of two: still bf16 values
    if stage == wl.SATTN:
        for im in w.images:
            im[:, 0:4, 0:8] = wl.bf16_round(im[:, 0:4, 0:8] * np.float32(0.05))
    else:
        w.ctx[:, :32] = wl.bf16_round(w.ctx[:, :32] * np.float32(0.05))
    # the inputs do reach the path: count the rows, from the oracle's own logits, in the key order of the patch batch
    late = 0
    for i in (0, len(res) - 1):
        z = np.asarray(w.images[i], dtype=np.float64)
        if stage == wl.SATTN:
            ut = op.split([ob.group_norm(z, p["gn_g"], p["gn_b"], cfg.G, cfg.eps)], 4, 4)      # patch-major token order
            late += _late_maximum_rows(ut @ p["wq"].astype(np.float64), ut @ p["wk"].astype(np.float64), 2)
        else:
            late += _late_maximum_rows(ob._tokens(z) @ p["wq"].astype(np.float64),
                                       w.ctx[i].astype(np.float64) @ p["wk"].astype(np.float64), 2)
    assert late > 100, late
    got = GpuRun(w).forward_images()
    ref, _ = _oracle(w)
    err = rel_err(got, ref)
    print(f"wide logits ({name}, {stage}): {late} late maxima in two images, rel err {err:.3e}")
    assert err < 2e-2


@pytest.mark.parametrize("stage", [wl.SATTN, wl.XATTN])
@pytest.mark.parametrize("name,res", WIDE, ids=[c[0] for c in WIDE])
def test_attention_extreme_logits(name, res, stage):
    """Logits far outside the range in which 2^logit can be formed without a softmax reference (the large query tile
    then has to run its second pass): every logit of head 0 is shifted by about +185 and every logit of head 1 by about
    -185 (base 2).  The shift is the same for all keys of a query, so the softmax, and with it the oracle's result, is
    that of the unshifted problem, and bf16 rounding cannot turn it into a different one: the last eight dimensions of
    every key are exactly 4, those of every query exactly +-32, and nothing else touches these dimensions.  (A constant
    input channel does it: a GroupNorm group of constant channels gives beta, for the text keys a constant column.)"""
    C, d = 128, 64
    cfg = wl.custom_config(res, (4, 4), C=C, G=32, heads=2, stages=(stage,), dtype="bf16", ctx_len=77, ctx_dim=64, seed=79)
    w = wl.make_workload(cfg)
    p = w.params[0]
    tail = np.concatenate([np.arange(56, 64), np.arange(64 + 56, 128)])              # last eight dimensions of both heads
    p["wq"][:, tail] = 0.0
    p["wk"][:, tail] = 0.0
    p["wq"][0, 56:64] = 32.0
    p["wq"][0, 64 + 56:128] = -32.0
    p["wk"][0, tail] = 4.0
    if stage == wl.SATTN:
        for im in w.images:
            im[0:4] = 1.0                                        # group 0 constant: normalised to exactly beta
        p["gn_b"][0] = 1.0
        p["gn_b"][1:4] = 0.0
    else:
        for im in w.images:
            im[0] = 1.0                                          # the queries come from x itself
        w.ctx[:, :, 0] = 1.0
    # the shift, from the oracle's own logits
    z = np.asarray(w.images[0], dtype=np.float64)
    if stage == wl.SATTN:
        ut = ob._tokens(ob.group_norm(z, p["gn_g"], p["gn_b"], cfg.G, cfg.eps))
        Q, K = ut @ p["wq"].astype(np.float64), ut @ p["wk"].astype(np.float64)
    else:
        Q, K = ob._tokens(z) @ p["wq"].astype(np.float64), w.ctx[0].astype(np.float64) @ p["wk"].astype(np.float64)
    for h, sign in ((0, 1.0), (1, -1.0)):
        S2 = (Q[:, h * d:(h + 1) * d] @ K[:, h * d:(h + 1) * d].T) * (LOG2E / np.sqrt(d))
        assert (sign * S2).min() > 150.0, (h, S2.min(), S2.max())
    got = GpuRun(w).forward_images()
    ref, _ = _oracle(w)
    err = rel_err(got, ref)
    print(f"extreme logits ({name}, {stage}): rel err {err:.3e}")
    assert err < 2e-2


@pytest.mark.parametrize("offset", [30.0, -30.0, 1000.0])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("stages", [(wl.RES2,), (wl.SATTN,), (wl.RES1, wl.SATTN)])
def test_groupnorm_offset_input(stages, dtype, offset):
    """Inputs with mean = 30 (fp32 also 1,000) standard deviations: a variance formed as E[x^2] - mean^2 in fp32 would lose
    four (seven) digits.  bf16 inputs carry eight bits: an offset of 1,000 would leave nothing of them to normalise."""
    if dtype == "bf16" and offset > 100.0:
        pytest.skip("bf16 storage holds no deviation of order 1 at 1,000")
    cfg = wl.custom_config([(16, 16), (8, 24), (8, 8)], (8, 8), C=64, G=8, heads=1, stages=stages, dtype=dtype, seed=51)
    w = wl.make_workload(cfg)
    rd = wl.bf16_round if dtype == "bf16" else (lambda a: a)
    w.images = [rd(im + np.float32(offset)) for im in w.images]
    got = GpuRun(w).forward_images()
    ref, _ = _oracle(w)
    err = rel_err(got, ref)
    print(f"offset {offset} {stages} {dtype}: rel err {err:.3e}")
    assert err < tolerance(dtype)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_groupnorm_offset_second_norm_and_reuse(dtype):
    """The second norm of the residual block takes its partial sums from the first convolution's epilogue (no mask) or
    from a pass over cached and fresh patches (mask): a large convolution bias shifts that tensor's mean to about 30
    standard deviations (fp32).  In bf16 that tensor is STORED with eight bits of mantissa, so an offset of 30 would
    quantise it in steps of 1/8 of its standard deviation whatever the statistics do; the bf16 case uses 4."""
    cfg = wl.custom_config([(16, 16), (8, 24), (8, 8)], (8, 8), C=64, G=8, heads=1, stages=(wl.RES2,), dtype=dtype,
                           reuse_p=0.4, seed=52)
    w = wl.make_workload(cfg)
    rd = wl.bf16_round if dtype == "bf16" else (lambda a: a)
    off = np.float32(30.0 if dtype == "f32" else 4.0)
    w.params[0]["conv_a_b"] = rd(w.params[0]["conv_a_b"] + off)
    w.cache["0.h1"] = [rd(c + off) for c in w.cache["0.h1"]]
    run = GpuRun(w)
    got = run.forward_images()
    ref, _ = _oracle(w)
    assert rel_err(got, ref) < tolerance(dtype)
    run.load_cache()
    got = run.forward_images(reuse=w.reuse)
    ref, _ = _oracle(w, reuse=w.reuse, cache=w.cache)
    assert rel_err(got, ref) < tolerance(dtype)


def test_groupnorm_offset_mfma_width():
    """The same at a width that takes the MFMA convolution (its epilogue leaves the second norm's partial sums)."""
    cfg = wl.custom_config([(32, 32), (16, 48), (16, 16)], (16, 16), C=320, G=32, heads=5, stages=(wl.RES2,), dtype="bf16",
                           seed=53)
    w = wl.make_workload(cfg)
    w.images = [wl.bf16_round(im + np.float32(30.0)) for im in w.images]
    w.params[0]["conv_a_b"] = wl.bf16_round(w.params[0]["conv_a_b"] + np.float32(4.0))
    got = GpuRun(w).forward_images()
    ref, _ = _oracle(w)
    err = rel_err(got, ref)
    print(f"offset, C = 320: rel err {err:.3e}")
    assert err < 2e-2
