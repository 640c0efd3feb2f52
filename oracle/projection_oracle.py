"""CPU oracle of the block-to-patch projection -- TEST INFRASTRUCTURE ONLY.

Sec. 3.3.1 of the CodecSight paper (the paragraph on mapping codec changes to ViT patches): block
rectangles are given in source-frame pixels, patches in model-input pixels; rescale the rectangles
and give every patch the strongest motion (Eq. 1) found among the blocks that land on it.
Sec. 3.3.2: a patch touched by an intra-coded block carries the intra flag.

Written as the definition: for every patch, test every block for overlap, take the maximum.
Geometry is exact (integer cross-multiplication, no floating point).  Shares nothing with the HIP
path.  Pinned in tests/test_projection_pins.py by hand-worked examples (tests/golden/), a brute-force
painter on a fine common grid, aligned-geometry special cases and invariants.

Readings (the paper leaves them open):
  * scaling is a plain resize: source (x, y) -> (x * in_w / src_w, y * in_h / src_h);
  * "overlap" is an intersection of positive area between the projected footprint
    [x sx, (x+w) sx) x [y sy, (y+h) sy) and the patch [c p, (c+1) p) x [r p, (r+1) p);
    footprints are clipped to the source frame;
  * the patch carries the motion vector of the winning block (the scoring step compares its
    squared magnitude); among blocks of equal magnitude the lexicographically largest (dx, dy)
    wins, which makes the result independent of block order;
  * intra-coded blocks have no motion vector and take no part in the maximum;
  * a patch no inter block overlaps gets (0, 0).
"""
from __future__ import annotations

import numpy as np

BLOCK_INTRA = 1      # bit 0 of a block's flags

BLOCK_DTYPE = np.dtype([("x", "<u2"), ("y", "<u2"), ("w", "<u2"), ("h", "<u2"),
                        ("dx", "<i2"), ("dy", "<i2"), ("flags", "<u4")])


def overlaps_1d(start, length, limit, scale_num, scale_den, patch, index):
    """Does [start, start+length) clipped to [0, limit), scaled by scale_num/scale_den, meet patch
    cell [index*patch, (index+1)*patch) in more than a point?  Integer arrays in, bool array out."""
    lo = np.minimum(start.astype(np.int64), limit)
    hi = np.minimum(start.astype(np.int64) + length.astype(np.int64), limit)
    # lo*s < (index+1)*patch   and   hi*s > index*patch,   s = scale_num / scale_den
    return (lo * scale_num < (index + 1) * patch * scale_den) & (hi * scale_num > index * patch * scale_den) & (hi > lo)


def project_frame(blocks, src_w, src_h, in_w, in_h, patch, grid_h, grid_w):
    """One frame.  blocks: structured array (BLOCK_DTYPE).  Returns (mv [P,2] int16, intra [P] uint8)."""
    mv = np.zeros((grid_h * grid_w, 2), np.int16)
    intra = np.zeros(grid_h * grid_w, np.uint8)
    is_intra = (blocks["flags"] & BLOCK_INTRA) != 0
    dx = blocks["dx"].astype(np.int64)
    dy = blocks["dy"].astype(np.int64)
    v_sq = dx * dx + dy * dy                                   # Eq. 1, squared
    for r in range(grid_h):
        in_row = overlaps_1d(blocks["y"], blocks["h"], src_h, in_h, src_h, patch, r)
        for c in range(grid_w):
            hit = in_row & overlaps_1d(blocks["x"], blocks["w"], src_w, in_w, src_w, patch, c)
            if (hit & is_intra).any():
                intra[r * grid_w + c] = 1
            inter = np.flatnonzero(hit & ~is_intra)
            if inter.size:
                best = max(inter, key=lambda m: (int(v_sq[m]), int(dx[m]), int(dy[m])))
                mv[r * grid_w + c] = (dx[best], dy[best])
    return mv, intra


def project_blocks(blocks, cu_blocks, src_w, src_h, in_w, in_h, patch, grid_h, grid_w):
    """A batch of frames: blocks of frame f are blocks[cu_blocks[f]:cu_blocks[f+1]].
    Returns (mv [F,P,2] int16, intra [F,P] uint8): the inputs of the scoring step."""
    n_frames = len(cu_blocks) - 1
    mv = np.zeros((n_frames, grid_h * grid_w, 2), np.int16)
    intra = np.zeros((n_frames, grid_h * grid_w), np.uint8)
    for f in range(n_frames):
        mv[f], intra[f] = project_frame(blocks[cu_blocks[f]:cu_blocks[f + 1]], src_w, src_h, in_w, in_h,
                                        patch, grid_h, grid_w)
    return mv, intra
