"""CPU oracle of the resolution changes between two levels of the first model's network.

TEST INFRASTRUCTURE ONLY (imported by tests; never by the product path; shares no code with it).

Two operators on ONE whole image u[C, H, W] (float64), written from their plain definitions:

* down2: 3x3 convolution with stride 2 and zero padding 1 (cross-correlation, like the block's convolution):
      out[co, oy, ox] = b[co] + sum_{ci, ty, tx} W[co, ci, ty, tx] * pad(u)[ci, 2*oy + ty, 2*ox + tx],
  pad(u) = u with a ring of zeros, so the taps of output pixel (oy, ox) are centred on input pixel (2*oy, 2*ox);
  H and W even, output [C_out, H/2, W/2].
* up2: every pixel repeated 2 x 2 (nearest neighbour), then the stride-1 3x3 convolution with zero padding 1;
  output [C_out, 2H, 2W].

Under patching both keep the patch grid: a patch of ph x pw pixels becomes one of ph/2 x pw/2 (2ph x 2pw), which is
why the paper's patch-size rule (greatest common divisor of the resolutions) survives a level change; the halo of the
convolution comes from the neighbour patches as in the block ("Patch-Tailored Diffusion Operators").
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def down2(u: np.ndarray, W: np.ndarray, b: np.ndarray) -> np.ndarray:
    C, H, Wd = u.shape
    assert H % 2 == 0 and Wd % 2 == 0
    Co = W.shape[0]
    pad = np.zeros((C, H + 2, Wd + 2), dtype=F64)
    pad[:, 1:-1, 1:-1] = u
    out = np.zeros((Co, H // 2, Wd // 2), dtype=F64)
    for ty in range(3):
        for tx in range(3):
            # pad[ci, 2*oy + ty, 2*ox + tx] for all (oy, ox)
            view = pad[:, ty:ty + H:2, tx:tx + Wd:2]
            out += np.einsum("oc,cyx->oyx", W[:, :, ty, tx].astype(F64), view)
    return out + b.astype(F64)[:, None, None]


def up2(u: np.ndarray, W: np.ndarray, b: np.ndarray) -> np.ndarray:
    C, H, Wd = u.shape
    Co = W.shape[0]
    big = np.zeros((C, 2 * H, 2 * Wd), dtype=F64)
    for a in range(2):
        for c in range(2):
            big[:, a::2, c::2] = u                       # pixel (y, x) fills (2y + a, 2x + c)
    pad = np.zeros((C, 2 * H + 2, 2 * Wd + 2), dtype=F64)
    pad[:, 1:-1, 1:-1] = big
    out = np.zeros((Co, 2 * H, 2 * Wd), dtype=F64)
    for ty in range(3):
        for tx in range(3):
            out += np.einsum("oc,cyx->oyx", W[:, :, ty, tx].astype(F64), pad[:, ty:ty + 2 * H, tx:tx + 2 * Wd])
    return out + b.astype(F64)[:, None, None]
