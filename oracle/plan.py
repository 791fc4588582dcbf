"""CPU oracle of the patch planner tables and of split / reassembly.

TEST INFRASTRUCTURE ONLY (imported by tests, the smoke check and the benchmark's
CPU-baseline leg; never by the product path; shares no code with it).

Compressed Sparse Patch format (section "Compressed Sparse Patch Format"): requests
are reordered by resolution, the patches of one image are stored densely, a
RequestOffset array gives the first patch of every request, every patch carries the
index of its request, and resolution offsets delimit requests of equal resolution.
Neighbour metadata (section "Patch-Tailored Diffusion Operators"): each patch records
its adjacent patches at split time, absent neighbours mean zero fill.

Everything here is derived from ABSOLUTE pixel coordinates by exhaustive lookup:
every token is placed at (request slot, Y, X) and neighbours / halo sources are
found by looking that coordinate up, so no index formula of the HIP planner is
repeated.

Readings where the paper is silent (figure of the worked example is not available):
  * sort ascending by (H, W), stable in arrival order; perm[s] = caller index of slot s
  * patches of an image in row-major order over its patch grid
  * neighbour order NW, N, NE, W, E, SW, S, SE; -1 = absent
  * halo ring order: top row x=-1..pw, bottom row x=-1..pw, left column y=0..ph-1,
    right column y=0..ph-1; entries are global token ids, -1 = outside the image
  * token id = patch*ph*pw + y*pw + x
  * patch size (0, 0) means the greatest common divisor of all heights resp. widths
  * text_len > 0 (joint text-image attention of the paper's second model, section "Patch-based Self-Attention
    Module": every image token attends to its own request's tokens): the text tokens of a request ride along as
    ceil(text_len / (ph*pw)) extra patches placed behind its image patches, grid position (-1, k), no neighbours,
    no halo; seq_len[s] = H*W + text_len counts the valid tokens of slot s (the padding of the last text patch
    lies behind them), so a request's key set is the token range [cu_seqlens[s], cu_seqlens[s] + seq_len[s])
"""
from __future__ import annotations

import math
from functools import reduce
from typing import Dict, List, Sequence, Tuple

import numpy as np

NEIGHBOUR_ORDER = [(-1, -1), (-1, 0), (-1, 1), (0, -1), (0, 1), (1, -1), (1, 0), (1, 1)]


def plan_tables(resolutions: Sequence[Tuple[int, int]], ph: int = 0, pw: int = 0, text_len: int = 0) -> Dict[str, np.ndarray]:
    n = len(resolutions)
    if ph == 0 and pw == 0:
        ph = reduce(math.gcd, [h for h, _ in resolutions])
        pw = reduce(math.gcd, [w for _, w in resolutions])
    perm = sorted(range(n), key=lambda i: (resolutions[i][0], resolutions[i][1], i))
    res_sorted = [resolutions[i] for i in perm]

    # place every patch and every token at absolute coordinates
    patch_at: Dict[Tuple[int, int, int], int] = {}      # (slot, r, c) -> patch id
    token_at: Dict[Tuple[int, int, int], int] = {}      # (slot, Y, X) -> token id
    owner: List[int] = []
    rc: List[Tuple[int, int]] = []
    request_offset = [0]
    for s, (H, W) in enumerate(res_sorted):
        for r in range(H // ph):
            for c in range(W // pw):
                p = len(owner)
                patch_at[(s, r, c)] = p
                owner.append(s)
                rc.append((r, c))
                for y in range(ph):
                    for x in range(pw):
                        token_at[(s, r * ph + y, c * pw + x)] = p * ph * pw + y * pw + x
        for k in range(-(-text_len // (ph * pw))):              # text patches: off the grid, found by nobody
            owner.append(s)
            rc.append((-1, k))
        request_offset.append(len(owner))
    P = len(owner)

    neighbour = np.full((P, 8), -1, dtype=np.int32)
    ring = [(-1, x) for x in range(-1, pw + 1)] + [(ph, x) for x in range(-1, pw + 1)] \
        + [(y, -1) for y in range(ph)] + [(y, pw) for y in range(ph)]
    halo_src = np.full((P, len(ring)), -1, dtype=np.int32)
    for p in range(P):
        s, (r, c) = owner[p], rc[p]
        if r < 0:
            continue
        for k, (dy, dx) in enumerate(NEIGHBOUR_ORDER):
            neighbour[p, k] = patch_at.get((s, r + dy, c + dx), -1)
        for k, (y, x) in enumerate(ring):
            halo_src[p, k] = token_at.get((s, r * ph + y, c * pw + x), -1)

    res_hw: List[Tuple[int, int]] = []
    res_offset: List[int] = []
    for s, hw in enumerate(res_sorted):
        if not res_hw or res_hw[-1] != hw:
            res_hw.append(hw)
            res_offset.append(s)
    res_offset.append(n)
    return {
        "ph": ph, "pw": pw, "P": P, "T": P * ph * pw,
        "perm": np.array(perm, dtype=np.int32),
        "request_offset": np.array(request_offset, dtype=np.int32),
        "res_offset": np.array(res_offset, dtype=np.int32),
        "res_hw": np.array(res_hw, dtype=np.int32).reshape(-1, 2),
        "patch_owner": np.array(owner, dtype=np.int32),
        "patch_rc": np.array(rc, dtype=np.int32).reshape(-1, 2),
        "neighbour": neighbour,
        "halo_src": halo_src,
        "cu_seqlens": np.array(request_offset, dtype=np.int32) * (ph * pw),
        "seq_len": np.array([H * W + text_len for H, W in res_sorted], dtype=np.int32),
    }


def split(images: Sequence[np.ndarray], ph: int, pw: int) -> np.ndarray:
    """Per-image [C, H, W] arrays (caller order) -> patch-major token matrix x[T, C] by coordinates."""
    res = [im.shape[1:] for im in images]
    n = len(images)
    perm = sorted(range(n), key=lambda i: (res[i][0], res[i][1], i))
    rows = []
    for i in perm:
        im = images[i]
        C, H, W = im.shape
        for r in range(H // ph):
            for c in range(W // pw):
                blk = im[:, r * ph:(r + 1) * ph, c * pw:(c + 1) * pw]      # [C, ph, pw]
                rows.append(blk.reshape(C, ph * pw).T)
    return np.concatenate(rows, axis=0)


def reassemble(x: np.ndarray, resolutions: Sequence[Tuple[int, int]], ph: int, pw: int) -> List[np.ndarray]:
    """Patch-major x[T, C] -> per-image [C, H, W] arrays in caller order."""
    n = len(resolutions)
    perm = sorted(range(n), key=lambda i: (resolutions[i][0], resolutions[i][1], i))
    C = x.shape[1]
    out: List[np.ndarray] = [None] * n
    t = 0
    for i in perm:
        H, W = resolutions[i]
        im = np.empty((C, H, W), dtype=x.dtype)
        for r in range(H // ph):
            for c in range(W // pw):
                im[:, r * ph:(r + 1) * ph, c * pw:(c + 1) * pw] = x[t:t + ph * pw].T.reshape(C, ph, pw)
                t += ph * pw
        out[i] = im
    return out


def text_scatter(x: np.ndarray, text: np.ndarray, resolutions: Sequence[Tuple[int, int]], ph: int, pw: int) -> np.ndarray:
    """text [n, L, C] (caller order) into the text patches of the joint token matrix x[T, C] (copy returned); the
    padding rows of the last text patch become zero."""
    L = text.shape[1]
    t = plan_tables(resolutions, ph, pw, L)
    out = np.array(x, copy=True)
    S = ph * pw
    for s, i in enumerate(t["perm"]):
        H, W = resolutions[i]
        first = int(t["cu_seqlens"][s]) + H * W
        end = int(t["cu_seqlens"][s + 1])
        out[first:end] = 0
        out[first:first + L] = text[i]
    return out


def text_gather(x: np.ndarray, L: int, resolutions: Sequence[Tuple[int, int]], ph: int, pw: int) -> np.ndarray:
    """The text tokens of every request out of the joint token matrix: [n, L, C] in caller order."""
    t = plan_tables(resolutions, ph, pw, L)
    out = np.empty((len(resolutions), L, x.shape[1]), dtype=x.dtype)
    for s, i in enumerate(t["perm"]):
        H, W = resolutions[i]
        first = int(t["cu_seqlens"][s]) + H * W
        out[i] = x[first:first + L]
    return out
