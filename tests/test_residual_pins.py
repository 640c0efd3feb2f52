"""Pins of the residual-proxy oracle against things other than itself (CPU only): a hand-worked
example, closed forms, a per-pixel pure-Python loop with rational patch assignment, and the link
to the block residual of Eq. 2.  Each test names the mistake it would catch."""
import os
from fractions import Fraction

import numpy as np

from oracle import residual_oracle as ro

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "residual_proxy_example.txt")


def test_hand_worked_example():
    # vector sign or direction, x/y swapped, rounding of quarter pixels, edge handling, the 1/256 unit
    rows = {"prev": [], "cur": []}
    for line in open(GOLDEN):
        key, *rest = (line.strip().split() or ["#"])
        if key == "geometry":
            w, h, in_w, in_h, patch, gh, gw, cell = (int(v) for v in rest)
        elif key in rows:
            rows[key].append([int(v) for v in rest])
        elif key == "field":
            field = np.asarray([int(v) for v in rest], np.int16).reshape(h // cell, w // cell, 2)
        elif key == "score":
            want = [int(v) for v in rest]
    cur, prev = np.asarray(rows["cur"], np.uint8), np.asarray(rows["prev"], np.uint8)
    assert cur.shape == (h, w)
    assert ro.residual_frame(cur, prev, field, cell, in_w, in_h, patch, gh, gw).tolist() == want


def _frames(rng, h, w):
    return rng.integers(0, 256, size=(h, w), dtype=np.uint8), rng.integers(0, 256, size=(h, w), dtype=np.uint8)


def test_constant_offset_scores_that_offset():
    # cur = prev + k with zero vectors: every patch scores exactly 256 k (a sum instead of a mean,
    # or a wrong pixel count, shows)
    rng = np.random.default_rng(21)
    prev = rng.integers(0, 200, size=(24, 40), dtype=np.uint8)
    field = np.zeros((6, 10, 2), np.int16)
    for k in (0, 1, 37):
        got = ro.residual_frame((prev + k).astype(np.uint8), prev, field, 4, 20, 12, 4, 3, 5)
        assert np.all(got == 256 * k)


def test_exact_translation_scores_zero_and_the_wrong_direction_does_not():
    # cur(x, y) = prev(x + 3, y - 2) with edge replication, field = (12, -8) quarter pixels
    rng = np.random.default_rng(22)
    h, w = 20, 32
    prev = rng.integers(0, 256, size=(h, w), dtype=np.uint8)
    ys, xs = np.meshgrid(np.arange(h), np.arange(w), indexing="ij")
    cur = prev[np.clip(ys - 2, 0, h - 1), np.clip(xs + 3, 0, w - 1)]
    field = np.zeros((5, 8, 2), np.int16)
    field[..., 0], field[..., 1] = 12, -8
    assert not ro.residual_frame(cur, prev, field, 4, 16, 10, 2, 5, 8).any()
    for bad in ((-12, 8), (-8, 12), (12, 8)):
        field[..., 0], field[..., 1] = bad
        assert ro.residual_frame(cur, prev, field, 4, 16, 10, 2, 5, 8).any()


def test_quarter_pixel_rounding():
    # offsets floor((d+2)/4): d = -6..6 -> -1 -1 -1 -1 0 0 0 0 1 1 1 1 2
    prev = np.arange(64, dtype=np.uint8).reshape(1, 64).repeat(4, axis=0) * 3
    want = [-1, -1, -1, -1, 0, 0, 0, 0, 1, 1, 1, 1, 2]
    for d, o in zip(range(-6, 7), want):
        field = np.zeros((1, 16, 2), np.int16)
        field[..., 0] = d
        pred = ro.predicted_frame(prev, field, 4)
        assert np.array_equal(pred[:, 8:56], prev[:, 8 + o:56 + o]), d


def _loops(cur, prev, field, cell, in_w, in_h, patch, gh, gw):
    h, w = cur.shape
    total, count = {}, {}
    for y in range(h):
        r = int(Fraction(y * in_h, h) / patch)              # floor of a non-negative rational
        for x in range(w):
            c = int(Fraction(x * in_w, w) / patch)
            if r >= gh or c >= gw:
                continue
            dx, dy = int(field[y // cell, x // cell, 0]), int(field[y // cell, x // cell, 1])
            ox, oy = (dx + 2) // 4, (dy + 2) // 4
            ref = int(prev[min(max(y + oy, 0), h - 1), min(max(x + ox, 0), w - 1)])
            total[(r, c)] = total.get((r, c), 0) + abs(int(cur[y, x]) - ref)
            count[(r, c)] = count.get((r, c), 0) + 1
    out = np.zeros(gh * gw, np.uint32)
    for (r, c), t in total.items():
        out[r * gw + c] = (256 * t) // count[(r, c)]
    return out


def test_against_pixel_loops_on_awkward_geometries():
    rng = np.random.default_rng(23)
    cases = [  # h, w, cell, in_w, in_h, patch, gh, gw
        (12, 20, 4, 15, 9, 3, 3, 5), (10, 30, 4, 20, 10, 5, 2, 4), (16, 16, 8, 28, 28, 7, 4, 4),
        (9, 13, 4, 26, 27, 9, 3, 3), (18, 31, 16, 14, 14, 7, 1, 1), (8, 8, 4, 16, 16, 1, 16, 16),
    ]
    for h, w, cell, in_w, in_h, patch, gh, gw in cases:
        cur, prev = _frames(rng, h, w)
        field = rng.integers(-40, 41, size=(-(-h // cell), -(-w // cell), 2)).astype(np.int16)
        got = ro.residual_frame(cur, prev, field, cell, in_w, in_h, patch, gh, gw)
        assert np.array_equal(got, _loops(cur, prev, field, cell, in_w, in_h, patch, gh, gw)), (h, w)


def test_score_is_the_block_residual_of_eq2_regrouped_by_patch():
    # aligned geometry (a patch = 2 x 2 blocks of 4 x 4 pixels): sum of the blocks' absolute
    # differences (Eq. 2) over the patch, divided by its pixel count, is the score
    rng = np.random.default_rng(24)
    h, w, cell = 16, 24, 4
    cur, prev = _frames(rng, h, w)
    field = rng.integers(-9, 10, size=(h // cell, w // cell, 2)).astype(np.int16)
    pred = ro.predicted_frame(prev, field, cell).astype(np.int64)
    sad = np.abs(cur.astype(np.int64) - pred).reshape(h // cell, cell, w // cell, cell).sum(axis=(1, 3))   # Eq. 2 per block
    per_patch = sad.reshape(2, 2, 3, 2).sum(axis=(1, 3))
    got = ro.residual_frame(cur, prev, field, cell, 12, 8, 4, 2, 3)
    assert np.array_equal(got.reshape(2, 3), (256 * per_patch) // 64)


def test_batch_is_frame_by_frame():
    rng = np.random.default_rng(25)
    cur = rng.integers(0, 256, size=(3, 8, 12), dtype=np.uint8)
    prev = rng.integers(0, 256, size=(3, 8, 12), dtype=np.uint8)
    field = rng.integers(-20, 21, size=(3, 2, 3, 2)).astype(np.int16)
    got = ro.residual_proxy(cur, prev, field, 4, 6, 4, 2, 2, 3)
    for f in range(3):
        assert np.array_equal(got[f], ro.residual_frame(cur[f], prev[f], field[f], 4, 6, 4, 2, 2, 3))
    assert ro.residual_proxy(cur[:0], prev[:0], field[:0], 4, 6, 4, 2, 2, 3).shape == (0, 6)
