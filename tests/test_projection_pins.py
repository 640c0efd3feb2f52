"""Pins of the block-to-patch projection oracle against things other than itself (CPU only).

Sources of truth: hand-worked examples (tests/golden/block_projection_example.txt), a brute-force
painter that rasterises every projected footprint on a fine grid common to source pixels and
patches (exact rationals), aligned geometries where the answer is the block's own vector, and
invariants the definition implies.  Each test names the mistake it would catch.
"""
import os
from fractions import Fraction

import numpy as np

from oracle import codecsight_oracle as oc
from oracle import projection_oracle as po

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "block_projection_example.txt")


def _blocks(rows):
    b = np.zeros(len(rows), po.BLOCK_DTYPE)
    for i, (x, y, w, h, dx, dy, flags) in enumerate(rows):
        b[i] = (x, y, w, h, dx, dy, flags)
    return b


def _golden_cases():
    cases, cur = [], None
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *rest = line.split()
        if key == "case":
            cur = dict(name=rest[0], blocks=[], mv=[], intra=[])
            cases.append(cur)
        elif key == "geometry":
            cur["geometry"] = [int(v) for v in rest]
        elif key == "block":
            cur["blocks"].append([int(v) for v in rest])
        elif key == "mv":
            cur["mv"].append([[int(v) for v in cell.split(",")] for cell in rest])
        elif key == "intra":
            cur["intra"].append([int(v) for v in rest])
    return cases


def test_hand_worked_examples():
    # wrong scaling direction, closed instead of half-open footprints (leaks over a shared edge),
    # min instead of max, intra blocks entering the maximum, the tie rule
    cases = _golden_cases()
    assert [c["name"] for c in cases] == ["A", "B"]
    for c in cases:
        src_w, src_h, in_w, in_h, patch, gh, gw = c["geometry"]
        mv, intra = po.project_frame(_blocks(c["blocks"]), src_w, src_h, in_w, in_h, patch, gh, gw)
        assert mv.reshape(gh, gw, 2).tolist() == c["mv"], c["name"]
        assert intra.reshape(gh, gw).tolist() == c["intra"], c["name"]


def _paint(blocks, src_w, src_h, in_w, in_h, patch, gh, gw):
    """Brute force: cut the model input into cells of 1/src_w x 1/src_h input pixels ... in exact
    rationals every source pixel column maps to [x*in_w/src_w, (x+1)*in_w/src_w); a source pixel
    belongs to every patch its image meets in more than a point.  Paint each block pixel by pixel."""
    best = {}
    intra = np.zeros((gh, gw), np.uint8)

    def cells(pix, n_src, n_in, n_grid):
        lo, hi = Fraction(pix * n_in, n_src), Fraction((pix + 1) * n_in, n_src)
        return [g for g in range(n_grid) if lo < (g + 1) * patch and hi > g * patch]

    col_of = [cells(x, src_w, in_w, gw) for x in range(src_w)]
    row_of = [cells(y, src_h, in_h, gh) for y in range(src_h)]
    for b in blocks:
        for y in range(int(b["y"]), min(int(b["y"]) + int(b["h"]), src_h)):
            for x in range(int(b["x"]), min(int(b["x"]) + int(b["w"]), src_w)):
                for r in row_of[y]:
                    for c in col_of[x]:
                        if b["flags"] & 1:
                            intra[r, c] = 1
                        else:
                            dx, dy = int(b["dx"]), int(b["dy"])
                            key = (dx * dx + dy * dy, dx, dy)
                            if (r, c) not in best or key > best[(r, c)]:
                                best[(r, c)] = key
    mv = np.zeros((gh, gw, 2), np.int16)
    for (r, c), key in best.items():
        mv[r, c] = key[1:]
    return mv.reshape(-1, 2), intra.reshape(-1)


def _random_blocks(rng, n, src_w, src_h, max_size, p_intra=0.1, spread=6):
    rows = []
    for _ in range(n):
        w, h = int(rng.integers(1, max_size + 1)), int(rng.integers(1, max_size + 1))
        x, y = int(rng.integers(0, src_w)), int(rng.integers(0, src_h))          # may stick out of the frame
        dx, dy = (int(v) for v in rng.integers(-spread, spread + 1, size=2))
        rows.append((x, y, w, h, dx, dy, int(rng.random() < p_intra)))
    return _blocks(rows)


def test_against_pixel_painter_on_awkward_scalings():
    # an off-by-one in either end of the patch range, transposed axes, a scaling that rounds
    rng = np.random.default_rng(11)
    geometries = [  # src_w, src_h, in_w, in_h, patch, gh, gw
        (30, 10, 20, 10, 5, 2, 4), (17, 23, 12, 18, 3, 6, 4), (40, 24, 28, 28, 7, 4, 4),
        (13, 9, 26, 27, 9, 3, 3),                    # upscaling
        (31, 19, 14, 14, 7, 2, 2), (25, 25, 20, 15, 5, 2, 3),   # grid smaller than the input: clipped
    ]
    for g in geometries:
        for trial in range(6):
            b = _random_blocks(rng, int(rng.integers(1, 14)), g[0], g[1], max(2, g[0] // 2))
            mv_w, intra_w = _paint(b, *g)
            mv_g, intra_g = po.project_frame(b, *g)
            assert np.array_equal(mv_g, mv_w), (g, trial)
            assert np.array_equal(intra_g, intra_w), (g, trial)


def test_aligned_geometry_returns_each_blocks_own_vector():
    # blocks that coincide with patches: the projection is the identity (any leak shows up)
    rng = np.random.default_rng(12)
    gh, gw, patch, k = 5, 7, 4, 3                      # source = input * 3
    vec = rng.integers(-50, 51, size=(gh * gw, 2))
    rows = [(c * patch * k, r * patch * k, patch * k, patch * k, int(vec[r * gw + c, 0]), int(vec[r * gw + c, 1]), 0)
            for r in range(gh) for c in range(gw)]
    order = rng.permutation(len(rows))
    mv, intra = po.project_frame(_blocks([rows[i] for i in order]), gw * patch * k, gh * patch * k,
                                 gw * patch, gh * patch, patch, gh, gw)
    assert np.array_equal(mv, vec.astype(np.int16)) and not intra.any()


def test_invariants_of_the_maximum():
    rng = np.random.default_rng(13)
    g = (96, 64, 56, 42, 14, 3, 4)
    b = _random_blocks(rng, 40, g[0], g[1], 24, spread=20)
    mv, intra = po.project_frame(b, *g)
    mag = (mv.astype(np.int64) ** 2).sum(1)
    # order of the blocks does not matter (the tie rule is part of the definition)
    mv_p, intra_p = po.project_frame(b[rng.permutation(b.size)], *g)
    assert np.array_equal(mv_p, mv) and np.array_equal(intra_p, intra)
    # one more block never lowers a patch's magnitude and never clears a flag
    extra = np.concatenate([b, _random_blocks(rng, 1, g[0], g[1], 40, spread=30)])
    mv_e, intra_e = po.project_frame(extra, *g)
    assert np.all((mv_e.astype(np.int64) ** 2).sum(1) >= mag) and np.all(intra_e >= intra)
    # a block over the whole frame with the largest vector wins everywhere
    full = np.concatenate([b, _blocks([(0, 0, g[0], g[1], 100, -100, 0)])])
    mv_f, _ = po.project_frame(full, *g)
    assert np.all(mv_f == np.asarray([100, -100], np.int16))
    # only intra blocks: no vectors, flags where they lie; nothing at all: zeros
    only_intra = b.copy()
    only_intra["flags"] = 1
    mv_i, intra_i = po.project_frame(only_intra, *g)
    assert not mv_i.any() and intra_i.any()
    mv_0, intra_0 = po.project_frame(b[:0], *g)
    assert not mv_0.any() and not intra_0.any()
    # a block with no area, or starting outside the frame, has no footprint
    ghost = _blocks([(10, 10, 0, 8, 90, 90, 0), (g[0], 0, 8, 8, 90, 90, 0), (0, g[1] + 3, 8, 8, 90, 90, 1)])
    mv_g, intra_g = po.project_frame(ghost, *g)
    assert not mv_g.any() and not intra_g.any()


def test_thresholding_the_maximum_is_an_or_over_blocks():
    # Eq. 3 on the projected magnitude == "some overlapping inter block moves at least tau":
    # the reason a maximum (not a mean or a sum) is the right reduction for the scoring step
    rng = np.random.default_rng(14)
    g = (80, 48, 40, 24, 8, 3, 5)
    b = _random_blocks(rng, 30, g[0], g[1], 20, p_intra=0.0, spread=8)
    mv, _ = po.project_frame(b, *g)
    tau_sq = 41
    kept = oc.patch_decision(mv, None, None, tau_sq, 0, False)
    for r in range(g[5]):
        for c in range(g[6]):
            hit = po.overlaps_1d(b["y"], b["h"], g[1], g[3], g[1], g[4], r) & \
                  po.overlaps_1d(b["x"], b["w"], g[0], g[2], g[0], g[4], c)
            moving = (b["dx"].astype(int) ** 2 + b["dy"].astype(int) ** 2 >= tau_sq) & hit
            assert bool(kept[r * g[6] + c]) == bool(moving.any())


def test_batch_splits_frames_at_their_offsets():
    rng = np.random.default_rng(15)
    g = (64, 32, 32, 16, 8, 2, 4)
    frames = [_random_blocks(rng, n, g[0], g[1], 16) for n in (5, 0, 9)]
    cu = np.concatenate([[0], np.cumsum([f.size for f in frames])]).astype(np.int32)
    mv, intra = po.project_blocks(np.concatenate(frames), cu, *g)
    for f, fb in enumerate(frames):
        mv_f, intra_f = po.project_frame(fb, *g)
        assert np.array_equal(mv[f], mv_f) and np.array_equal(intra[f], intra_f)
