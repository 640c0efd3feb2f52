"""CPU oracle of the residual proxy -- TEST INFRASTRUCTURE ONLY.

Sec. 4 (Codec Processing) of the CodecSight paper: the hardware decoder hands out no residuals, so
they are approximated from pixels: shift the previous decoded frame by the motion vectors, compare
it with the current frame, and score a patch by the average absolute pixel difference inside it
(the per-patch counterpart of the block residual of Eq. 2, used by the rescue rule of Eq. 4).

Written as the definition: build the prediction pixel by pixel, take absolute differences, average
over the pixels of each patch.  Integers throughout.  Shares nothing with the HIP path.  Pinned in
tests/test_residual_pins.py by a hand-worked example (tests/golden/), closed forms (constant
offset, exact translation), a pure-Python pixel loop with rational patch assignment, and the
agreement of Eq. 2 summed over a patch's blocks with the un-normalised score.

Readings (the paper leaves them open):
  * frames are 8-bit luma planes at source resolution;
  * motion vectors are in quarter pixels on a regular field of cell x cell pixel cells (the finest
    partition of the codec), pointing from the current pixel to its reference:
    prediction(x, y) = previous(x + ox, y + oy), (ox, oy) = vector rounded to whole pixels as
    floor((d + 2) / 4) (no sub-pixel interpolation), coordinates clamped to the frame (edge
    replication); intra cells are given a zero vector by the caller;
  * a source pixel belongs to the patch its top-left corner projects into under the plain resize
    of the projection step: column floor(x * in_w / (patch * src_w)), row likewise; pixels that
    fall outside the grid are ignored;
  * the score is returned in 1/256 grey levels, floor(256 * sum / n), so that the scoring step's
    integer threshold applies; a patch without pixels scores 0.
"""
from __future__ import annotations

import numpy as np


def predicted_frame(prev, mv_field, cell):
    """Motion-compensated prediction of one frame.  prev: uint8 [H, W]; mv_field: int16
    [ceil(H/cell), ceil(W/cell), 2] quarter-pixel (dx, dy)."""
    h, w = prev.shape
    ys, xs = np.meshgrid(np.arange(h), np.arange(w), indexing="ij")
    d = mv_field[ys // cell, xs // cell].astype(np.int64)
    ox = np.floor_divide(d[..., 0] + 2, 4)
    oy = np.floor_divide(d[..., 1] + 2, 4)
    return prev[np.clip(ys + oy, 0, h - 1), np.clip(xs + ox, 0, w - 1)]


def patch_of(n_src, n_in, patch, n_grid):
    """Patch index of every source pixel coordinate 0..n_src-1 along one axis (-1: outside)."""
    idx = (np.arange(n_src, dtype=np.int64) * n_in) // (patch * n_src)
    return np.where(idx < n_grid, idx, -1)


def residual_frame(cur, prev, mv_field, cell, in_w, in_h, patch, grid_h, grid_w):
    """One frame: uint32 [grid_h*grid_w], mean |cur - prediction| per patch in 1/256 grey levels."""
    h, w = cur.shape
    diff = np.abs(cur.astype(np.int64) - predicted_frame(prev, mv_field, cell).astype(np.int64))
    col, row = patch_of(w, in_w, patch, grid_w), patch_of(h, in_h, patch, grid_h)
    out = np.zeros(grid_h * grid_w, np.uint32)
    for r in range(grid_h):
        for c in range(grid_w):
            block = diff[row == r][:, col == c]
            if block.size:
                out[r * grid_w + c] = (256 * int(block.sum())) // block.size
    return out


def residual_proxy(cur, prev, mv_field, cell, in_w, in_h, patch, grid_h, grid_w):
    """A batch: cur, prev uint8 [F, H, W]; mv_field int16 [F, H/cell, W/cell, 2] -> uint32 [F, P]."""
    return np.stack([residual_frame(cur[f], prev[f], mv_field[f], cell, in_w, in_h, patch, grid_h, grid_w)
                     for f in range(cur.shape[0])]) if cur.shape[0] else np.zeros((0, grid_h * grid_w), np.uint32)
