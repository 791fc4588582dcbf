"""CPU oracle of the patch-cache manager pieces.

TEST INFRASTRUCTURE ONLY (imported by tests; never by the product path; shares no code with it).

Two things of the paper's patch-level cache outside the block itself:

* the feature the cache reuse predictor looks at (section "Patch-aware Caching Strategy", step 1: the new
  input is compared with the cache of the previous step, per patch; the implementation section names the
  similarity metric, the mean squared error): per patch, the mean over its ph*pw*C elements of (a - b)^2;
* the id bookkeeping of section "Batching Patches in Cache": every patch has a unique id, here
  (request id, patch row, patch column); comparing the ids submitted with the new batch against the ids held
  by the cache gives the Common Set (in both), the New Set (only in the input) and the Expired Set (only in
  the cache).

Both are written from absolute coordinates and dictionaries: the per-patch error is taken on slices of the
per-image NCHW arrays (no patch batch is formed), the sets by looking ids up.  The order of the per-patch
outputs is the plan order (requests ascending by (H, W), stable; patches row-major inside an image), which is
recomputed here with a plain sort.

Readings: a request keeps its resolution while it is in the system, so a Common request has the same patch
grid in both batches (anything else is an error); both batches use the same patch size.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

import numpy as np


def _plan_order(resolutions: Sequence[Tuple[int, int]]) -> List[int]:
    return sorted(range(len(resolutions)), key=lambda i: (resolutions[i][0], resolutions[i][1], i))


def patch_mse(a: Sequence[np.ndarray], b: Sequence[np.ndarray], ph: int, pw: int) -> np.ndarray:
    """a[i], b[i]: image i as [C][H][W] (caller order).  Returns fp64 [P] in plan order."""
    res = [(x.shape[1], x.shape[2]) for x in a]
    out: List[float] = []
    for i in _plan_order(res):
        H, W = res[i]
        for r in range(H // ph):
            for c in range(W // pw):
                da = np.asarray(a[i], dtype=np.float64)[:, r * ph:(r + 1) * ph, c * pw:(c + 1) * pw]
                db = np.asarray(b[i], dtype=np.float64)[:, r * ph:(r + 1) * ph, c * pw:(c + 1) * pw]
                out.append(float(np.mean((da - db) ** 2)))
    return np.asarray(out, dtype=np.float64)


def cache_sets(res_old: Sequence[Tuple[int, int]], ids_old: Sequence[int], res_new: Sequence[Tuple[int, int]],
               ids_new: Sequence[int], ph: int, pw: int) -> Dict[str, np.ndarray]:
    """Common / New / Expired sets of requests and the patch-level source table.

    req_src[i]   : caller index in the old batch of new request i (Common Set), -1 for the New Set
    expired[j]   : 1 if old request j is in the Expired Set
    patch_src[p] : old plan's patch index with the same (request id, row, column) as new patch p, else -1
    """
    assert len(set(ids_old)) == len(ids_old) and len(set(ids_new)) == len(ids_new), "ids must be unique"
    # ids held by the cache: (request id, r, c) -> old patch index, in old plan order
    held: Dict[Tuple[int, int, int], int] = {}
    p = 0
    for j in _plan_order(res_old):
        H, W = res_old[j]
        for r in range(H // ph):
            for c in range(W // pw):
                held[(ids_old[j], r, c)] = p
                p += 1
    where_old = {rid: j for j, rid in enumerate(ids_old)}
    req_src = np.full(len(ids_new), -1, dtype=np.int32)
    for i, rid in enumerate(ids_new):
        if rid in where_old:
            assert tuple(res_old[where_old[rid]]) == tuple(res_new[i]), "a request changed its resolution"
            req_src[i] = where_old[rid]
    expired = np.asarray([0 if rid in set(ids_new) else 1 for rid in ids_old], dtype=np.uint8)
    patch_src: List[int] = []
    for i in _plan_order(res_new):
        H, W = res_new[i]
        for r in range(H // ph):
            for c in range(W // pw):
                patch_src.append(held.get((ids_new[i], r, c), -1))
    return {"req_src": req_src, "expired": expired, "patch_src": np.asarray(patch_src, dtype=np.int32)}


def migrate(slot_old: np.ndarray, patch_src: np.ndarray, S: int, fill: np.ndarray) -> np.ndarray:
    """slot_old [T_old][C] token-major; returns [T_new][C]: patch p takes old patch patch_src[p], else keeps `fill`."""
    out = np.array(fill, copy=True)
    for p, q in enumerate(patch_src):
        if q >= 0:
            out[p * S:(p + 1) * S] = slot_old[q * S:(q + 1) * S]
    return out
