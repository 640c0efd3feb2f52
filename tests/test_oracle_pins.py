"""Pins of the CPU oracle against things other than itself (CPU only).

Each test names the mistake it would catch.  Sources of truth used here: the literal (unsquared,
floating-point) form of Eq. 1/3, hand-built frame sequences, complex-number rotation, the relative
position property of RoPE, a per-element pure-Python attention loop, torch's library attention,
and the transformers library's rotary helper.
"""
import itertools
import math

import numpy as np
import pytest

from oracle import codecsight_oracle as oc

I, P = oc.FRAME_I, oc.FRAME_P


def _meta(n_frames, n_patch, rng=None):
    mv = np.zeros((n_frames, n_patch, 2), np.int16)
    sad = np.zeros((n_frames, n_patch), np.uint32)
    if rng is not None:
        mv[:] = rng.integers(-40, 41, size=mv.shape)
        sad[:] = rng.integers(0, 2000, size=sad.shape)
    return mv, sad


def _run(mv, sad, ftype, cu, acc, gh, gw, g=1, tmv=17, tsad=401, res=True, intra=None):
    return oc.score_compact(mv, sad if res else None, intra, np.asarray(ftype, np.uint8),
                            np.asarray(cu, np.int32), acc, gh, gw, g, tmv, tsad, res)


# ------------------------------------------------------------------ (a) scoring / compaction
def test_zero_thresholds_keep_every_patch():
    # '>=' with tau = 0 holds for every vector, including the zero vector (a strict '>' fails here)
    rng = np.random.default_rng(1)
    mv, sad = _meta(6, 64, rng)
    mv[2] = 0
    sad[2] = 0
    keep, idx, off, _ = _run(mv, sad, [P] * 6, [0, 3, 6], np.zeros((2, 64), np.uint8), 8, 8,
                             tmv=0, tsad=0)
    assert keep.all()
    assert np.array_equal(idx, np.arange(6 * 64))
    assert np.array_equal(off, np.arange(7) * 64)


def test_i_frame_keeps_all_and_ignores_metadata_and_resets_state():
    rng = np.random.default_rng(2)
    mv, sad = _meta(3, 16)
    mv_g, sad_g = _meta(3, 16, rng)             # garbage in the I-frame's slot must not matter
    for m, s_ in ((mv, sad), (mv_g, sad_g)):
        m[0] = 0
        s_[0] = 0
        m[2] = 0
        s_[2] = 0
    acc0 = np.ones((1, 16), np.uint8)
    a = _run(mv, sad, [P, I, P], [0, 3], acc0, 4, 4)
    b = _run(mv_g, sad_g, [P, I, P], [0, 3], acc0, 4, 4)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    keep, idx, off, acc = a
    assert keep[0].all()          # carried-in accumulated state keeps everything in the first P
    assert keep[1].all()          # the I-frame itself
    assert not keep[2].any()      # I reset the state and its own full mask was not accumulated
    assert not acc.any()


def test_threshold_is_inclusive_and_euclidean():
    # literal Eq. 1/3: keep iff hypot(dx, dy) >= tau, checked over every small vector
    vals = range(-6, 7)
    vecs = np.array(list(itertools.product(vals, vals)), np.int16)
    n = vecs.shape[0]
    mv = vecs.reshape(1, n, 2)
    for tau in (0.0, 1.0, 4.0, 5.0, 4.25, 7.0):
        tau_sq = math.ceil(tau * tau - 1e-12)
        keep, *_ = _run(mv, None, [P], [0, 1], None, 1, n, tmv=tau_sq, res=False)
        want = np.array([math.hypot(int(x), int(y)) >= tau for x, y in vecs], np.uint8)
        assert np.array_equal(keep[0], want), tau
    # (3,4) sits exactly on tau = 5; (4,4) is above 5.65 > 5; (3,3) below
    keep, *_ = _run(np.array([[[3, 4], [4, 4], [3, 3], [-5, 0], [0, -4]]], np.int16), None,
                    [P], [0, 1], None, 1, 5, tmv=25, res=False)
    assert keep[0].tolist() == [1, 1, 0, 1, 0]


def test_squared_magnitude_does_not_overflow():
    mv = np.array([[[-32768, -32768], [32767, 32767], [-32768, 0]]], np.int16)
    keep, *_ = _run(mv, None, [P], [0, 1], None, 1, 3, tmv=2**31 - 1 + 2**30, res=False)
    # largest possible value 2*32768^2 = 2^31 = 2147483648 is below the threshold 3221225471
    assert keep[0].tolist() == [0, 0, 0]
    keep, *_ = _run(mv, None, [P], [0, 1], None, 1, 3, tmv=2**31, res=False)
    assert keep[0].tolist() == [1, 0, 0]       # 2*32767^2 = 2147352578 < 2^31; 32768^2 = 2^30


def test_residual_rescue_only_adds_and_only_when_enabled():
    rng = np.random.default_rng(3)
    mv, sad = _meta(4, 100, rng)
    base, *_ = _run(mv, sad, [P] * 4, [0, 4], None, 10, 10, res=False)
    resc, *_ = _run(mv, sad, [P] * 4, [0, 4], None, 10, 10, res=True, tsad=900)
    assert np.all(resc >= base) and resc.sum() > base.sum()
    # exactly the patches with small motion and large residual were added (inclusive '>=')
    v2 = (mv.astype(np.int64) ** 2).sum(-1)
    assert np.array_equal(resc.astype(bool) & ~base.astype(bool), (v2 < 17) & (sad >= 900))
    sad2 = np.full_like(sad, 899)
    sad2[0, 0] = 900
    mv0 = np.zeros_like(mv)
    r2, *_ = _run(mv0, sad2, [P] * 4, [0, 4], None, 10, 10, res=True, tsad=900)
    assert r2.sum() == 1 and r2[0, 0] == 1


def test_intra_patches_are_kept():
    mv, sad = _meta(1, 9)
    intra = np.zeros((1, 9), np.uint8)
    intra[0, 4] = 7
    keep, idx, off, _ = _run(mv, sad, [P], [0, 1], None, 3, 3, intra=intra)
    assert keep[0].tolist() == [0, 0, 0, 0, 1, 0, 0, 0, 0] and idx.tolist() == [4]


def test_monotone_in_thresholds():
    rng = np.random.default_rng(4)
    mv, sad = _meta(5, 64, rng)
    prev = None
    for tmv in (0, 5, 17, 100, 900, 4000):
        keep, *_ = _run(mv, sad, [P] * 5, [0, 5], np.zeros((1, 64), np.uint8), 8, 8, tmv=tmv,
                        tsad=1500)
        if prev is not None:
            assert np.all(keep <= prev)
        prev = keep
    prev = None
    for tsad in (0, 100, 500, 1000, 5000):
        keep, *_ = _run(mv, sad, [P] * 5, [0, 5], None, 8, 8, tmv=3000, tsad=tsad)
        if prev is not None:
            assert np.all(keep <= prev)
        prev = keep


def test_gop_accumulation_hand_sequence():
    # one stream, 4 patches; motion at patch 0 in frame 0, patch 2 in frame 1, nothing after
    mv, sad = _meta(7, 4)
    mv[0, 0] = (9, 0)
    mv[1, 2] = (0, 9)
    mv[5, 3] = (9, 9)
    ft = [P, P, P, I, P, P, P]
    keep, idx, off, acc = _run(mv, sad, ft, [0, 7], np.zeros((1, 4), np.uint8), 2, 2)
    assert keep.tolist() == [[1, 0, 0, 0], [1, 0, 1, 0], [1, 0, 1, 0],   # sticky inside the GOP
                             [1, 1, 1, 1],                               # I-frame
                             [0, 0, 0, 0], [0, 0, 0, 1], [0, 0, 0, 1]]   # reset, then sticky again
    assert acc.tolist() == [[0, 0, 0, 1]]
    assert idx.tolist() == [0, 4, 6, 8, 10, 12, 13, 14, 15, 23, 27]
    assert off.tolist() == [0, 1, 3, 5, 9, 9, 10, 11]
    # without accumulation the mask is the per-frame rule alone
    keep2, *_ = _run(mv, sad, ft, [0, 7], None, 2, 2)
    assert keep2.tolist() == [[1, 0, 0, 0], [0, 0, 1, 0], [0, 0, 0, 0], [1, 1, 1, 1],
                              [0, 0, 0, 0], [0, 0, 0, 1], [0, 0, 0, 0]]
    # accumulated mask is monotone between I-frames
    assert np.all(keep[1] >= keep[0]) and np.all(keep[2] >= keep[1]) and np.all(keep[6] >= keep[5])


def test_streams_do_not_share_state():
    mv, sad = _meta(4, 4)
    mv[0, 1] = (20, 0)                       # stream 0, first frame
    keep, idx, off, acc = _run(mv, sad, [P, P, P, P], [0, 2, 4], np.zeros((2, 4), np.uint8), 2, 2)
    assert keep.tolist() == [[0, 1, 0, 0], [0, 1, 0, 0], [0, 0, 0, 0], [0, 0, 0, 0]]
    assert acc.tolist() == [[0, 1, 0, 0], [0, 0, 0, 0]]
    # carried-in state belongs to its own stream
    acc_in = np.array([[0, 0, 0, 0], [1, 0, 0, 0]], np.uint8)
    keep, *_ = _run(mv, sad, [P, P, P, P], [0, 2, 4], acc_in, 2, 2)
    assert keep.tolist() == [[0, 1, 0, 0], [0, 1, 0, 0], [1, 0, 0, 0], [1, 0, 0, 0]]


def test_projection_groups_on_a_non_square_grid():
    # 4 x 6 patches, 2x2 groups -> 2 x 3 tokens; one patch at (row 1, col 4) -> token (0, 2)
    mv, sad = _meta(1, 24)
    mv[0, 1 * 6 + 4] = (30, 30)
    keep, idx, off, _ = _run(mv, sad, [P], [0, 1], None, 4, 6, g=2)
    assert keep.shape == (1, 6) and keep[0].tolist() == [0, 0, 1, 0, 0, 0]
    mv[0, 3 * 6 + 0] = (30, 30)             # patch (3, 0) -> token (1, 0)
    keep, idx, off, _ = _run(mv, sad, [P], [0, 1], None, 4, 6, g=2)
    assert keep[0].tolist() == [0, 0, 1, 1, 0, 0] and idx.tolist() == [2, 3]
    # accumulation stays at patch granularity: state returned per patch, not per token
    *_, acc = _run(mv, sad, [P], [0, 1], np.zeros((1, 24), np.uint8), 4, 6, g=2)
    assert acc.sum() == 2 and acc[0, 10] == 1 and acc[0, 18] == 1


def test_huge_thresholds_keep_nothing():
    rng = np.random.default_rng(5)
    mv, sad = _meta(3, 16, rng)
    keep, idx, off, _ = _run(mv, sad, [P] * 3, [0, 3], None, 4, 4, tmv=0xFFFFFFFF, tsad=0xFFFFFFFF)
    assert not keep.any() and idx.size == 0 and off.tolist() == [0, 0, 0, 0]


def test_brute_force_all_two_frame_2x2_grids():
    # every assignment of a small vector alphabet to 4 patches x 2 frames, against a per-patch
    # Python walk using the unsquared norm; checks order, offsets and the accumulated state
    alphabet = [(0, 0), (3, 0), (0, -4), (4, 1), (-3, -3), (5, 0)]
    rngs = np.random.default_rng(6)
    combos = list(itertools.product(range(len(alphabet)), repeat=4))
    picks = rngs.choice(len(combos), size=300, replace=False)
    for a in picks[:150]:
        for b in picks[150:160]:
            mv = np.array([[alphabet[i] for i in combos[a]], [alphabet[i] for i in combos[b]]],
                          np.int16)
            keep, idx, off, acc = _run(mv, None, [P, P], [0, 2], np.zeros((1, 4), np.uint8), 2, 2,
                                       tmv=17, res=False)
            state = [False] * 4
            want_idx = []
            for f in range(2):
                for i in range(4):
                    state[i] = state[i] or math.hypot(*alphabet[(combos[a], combos[b])[f][i]]) > 4.0
                    if state[i]:
                        want_idx.append(f * 4 + i)
            assert idx.tolist() == want_idx
            assert off.tolist() == [0, sum(1 for x in want_idx if x < 4), len(want_idx)]
            assert acc[0].astype(bool).tolist() == state
            assert np.all(keep.reshape(-1)[idx] == 1) and keep.sum() == idx.size


# ------------------------------------------------------------------ (b) rotation
def test_rotation_matches_complex_multiplication():
    rng = np.random.default_rng(10)
    d, base = 64, 1e4
    x = rng.normal(size=(7, d))
    pos = rng.integers(-3000, 3000, size=7)
    got = oc.rotate(x, pos, base, style=0)
    theta = np.array([base ** (-2.0 * i / d) for i in range(d // 2)])
    z = (x[:, : d // 2] + 1j * x[:, d // 2:]) * np.exp(1j * pos[:, None] * theta[None])
    assert np.allclose(got[:, : d // 2], z.real, atol=1e-12)
    assert np.allclose(got[:, d // 2:], z.imag, atol=1e-12)
    got_i = oc.rotate(x, pos, base, style=1)
    zi = (x[:, 0::2] + 1j * x[:, 1::2]) * np.exp(1j * pos[:, None] * theta[None])
    assert np.allclose(got_i[:, 0::2], zi.real, atol=1e-12)
    assert np.allclose(got_i[:, 1::2], zi.imag, atol=1e-12)


def test_rotation_known_values():
    # theta_0 = 1 for any base: a quarter turn sends (1, 0) to (0, 1)  (sign convention)
    out = oc.rotate(np.array([[1.0, 0.0]]), np.array([math.pi / 2]), 123.0)
    assert np.allclose(out, [[0.0, 1.0]], atol=1e-15)
    # d = 4, base 1e4: theta_1 = 1e4^(-2/4) = 0.01; position 100 turns pair 1 by exactly 1 rad
    out = oc.rotate(np.array([[0.0, 1.0, 0.0, 0.0]]), np.array([100]), 1e4)
    assert np.allclose(out, [[0.0, math.cos(1.0), 0.0, math.sin(1.0)]], atol=1e-14)
    out = oc.rotate(np.array([[0.0, 0.0, 1.0, 0.0]]), np.array([100]), 1e4, style=1)
    assert np.allclose(out, [[0.0, 0.0, math.cos(1.0), math.sin(1.0)]], atol=1e-14)
    assert np.allclose(oc.rope_frequencies(128, 1e6)[[0, 32, 63]],
                       [1.0, 1e6 ** -0.5, 1e6 ** (-126.0 / 128.0)], rtol=1e-14)


def test_correction_equals_recomputation_at_the_new_position():
    # Eq. 6: R(p_new) R(p_old)^-1 K_old == key computed at p_new
    rng = np.random.default_rng(11)
    for d, base, style in ((64, 1e4, 0), (128, 1e6, 0), (128, 1e6, 1)):
        k_raw = rng.normal(size=(200, d))
        p_old = rng.integers(0, 20001, size=200)
        delta = rng.integers(-2392, 2393, size=200)
        cached = oc.rotate(k_raw, p_old, base, style)
        assert np.allclose(oc.rotate(cached, delta, base, style),
                           oc.rotate(k_raw, p_old + delta, base, style), atol=1e-10)


def test_rotation_group_properties_and_relative_position():
    rng = np.random.default_rng(12)
    d, base = 128, 1e6
    x = rng.normal(size=(50, d))
    a = rng.integers(-2000, 2000, size=50)
    b = rng.integers(-2000, 2000, size=50)
    assert np.array_equal(oc.rotate(x, np.zeros(50), base), x)
    assert np.allclose(oc.rotate(oc.rotate(x, a, base), -a, base), x, atol=1e-11)
    assert np.allclose(oc.rotate(oc.rotate(x, a, base), b, base), oc.rotate(x, a + b, base), atol=1e-10)
    y = oc.rotate(x, a, base)
    assert np.allclose(x[:, :64] ** 2 + x[:, 64:] ** 2, y[:, :64] ** 2 + y[:, 64:] ** 2, atol=1e-11)
    q = rng.normal(size=(50, d))
    lhs = (oc.rotate(q, a, base) * oc.rotate(x, b, base)).sum(-1)
    rhs = (oc.rotate(q, a - b, base) * x).sum(-1)
    assert np.allclose(lhs, rhs, atol=1e-9)


def test_rotation_against_transformers_rotary_helper():
    torch = pytest.importorskip("torch")
    mod = pytest.importorskip("transformers.models.llama.modeling_llama")
    d, base = 64, 1e4
    rng = np.random.default_rng(13)
    x = rng.normal(size=(1, 1, 9, d))
    pos = np.arange(9) * 37
    inv = 1.0 / (base ** (np.arange(0, d, 2, dtype=np.float64) / d))
    ang = pos[:, None] * inv[None]
    emb = np.concatenate([ang, ang], axis=-1)
    cos, sin = torch.from_numpy(np.cos(emb))[None], torch.from_numpy(np.sin(emb))[None]
    xt = torch.from_numpy(x)
    want, _ = mod.apply_rotary_pos_emb(xt, xt, cos, sin)
    got = oc.rotate(x[0, 0], pos, base, style=0)
    assert np.allclose(got, want[0, 0].numpy(), atol=1e-12)


def test_rerotate_on_a_pool_moves_the_right_rows_and_leaves_values_alone():
    rng = np.random.default_rng(14)
    n_layers, n_slots, n_heads, d, base = 3, 40, 2, 16, 1e4
    k = rng.normal(size=(n_layers, n_slots, n_heads, d)).astype(np.float32)
    v = rng.normal(size=(n_layers, n_slots, n_heads, d)).astype(np.float32)
    src = np.array([5, 9, 30], np.int32)
    dst = np.array([1, 2, 3], np.int32)
    delta = np.array([-256, 7, 0], np.int32)
    k_rows, v_rows = oc.rerotate(k, v, src, dst, delta, base)
    assert k_rows.shape == (3, n_layers, n_heads, d)
    for r in range(3):
        for l in range(n_layers):
            for h in range(n_heads):
                want = oc.rotate(k[l, src[r], h][None].astype(np.float64), delta[r:r + 1], base)[0]
                assert np.allclose(k_rows[r, l, h], want, atol=1e-13)
                assert np.array_equal(v_rows[r, l, h], v[l, src[r], h].astype(np.float64))
    assert np.array_equal(k_rows[2], np.transpose(k[:, 30], (0, 1, 2)).astype(np.float64))
    k_rows2, v_none = oc.rerotate(k, None, src, None, delta, base)
    assert v_none is None and np.array_equal(k_rows2, k_rows)


# ------------------------------------------------------------------ multi-axis RoPE (Sec. 3.4.2)
def _sections_axis_map(sections):
    return np.concatenate([np.full(n, a, np.int64) for a, n in enumerate(sections)])


def test_axes_rotation_known_values_and_untouched_pairs():
    # d = 4, base 1e4: theta = (1, 0.01); pair 0 follows h, pair 1 follows w; position (t,h,w) = (7, 2, 50)
    x = np.array([1.0, 0.0, 0.0, 1.0])                    # half-split pairs: (x0, x2), (x1, x3)
    got = oc.rotate_axes(x, np.array([7, 2, 50]), np.array([1, 2]), 1e4, style=0)
    assert np.allclose(got, [math.cos(2.0), -math.sin(0.5), math.sin(2.0), math.cos(0.5)], atol=1e-15)
    # a shift along t only leaves the pairs of the other axes exactly as they were
    rng = np.random.default_rng(21)
    d = 16
    axis = _sections_axis_map([2, 3, 3])
    y = rng.normal(size=(5, d))
    z = oc.rotate_axes(y, np.array([-256, 0, 0]), axis, 1e6)
    ia, ib = np.arange(d // 2), np.arange(d // 2) + d // 2
    keep = axis != 0
    assert np.array_equal(z[:, ia[keep]], y[:, ia[keep]]) and np.array_equal(z[:, ib[keep]], y[:, ib[keep]])
    assert not np.allclose(z[:, ia[~keep]], y[:, ia[~keep]])


def test_axes_rotation_with_one_axis_is_plain_rope():
    rng = np.random.default_rng(22)
    d, base = 32, 1e4
    x = rng.normal(size=(6, d))
    pos = rng.integers(-3000, 3000, size=6)
    for a in range(3):
        pos3 = rng.integers(-99, 99, size=(6, 3))
        pos3[:, a] = pos
        for style in (0, 1):
            got = oc.rotate_axes(x, pos3, np.full(d // 2, a), base, style)
            assert np.allclose(got, oc.rotate(x, pos, base, style), atol=1e-12)


def test_axes_correction_equals_recomputation_and_keeps_relative_scores():
    rng = np.random.default_rng(23)
    d, base = 32, 1e6
    axis = _sections_axis_map([4, 6, 6])
    k_raw, q_raw = rng.normal(size=(9, d)), rng.normal(size=(9, d))
    p_old = rng.integers(0, 4000, size=(9, 3))
    p_new = p_old + rng.integers(-2500, 2500, size=(9, 3))
    for style in (0, 1):
        cached = oc.rotate_axes(k_raw, p_old, axis, base, style)
        fixed = oc.rotate_axes(cached, p_new - p_old, axis, base, style)          # Eq. 6
        assert np.allclose(fixed, oc.rotate_axes(k_raw, p_new, axis, base, style), atol=1e-9)
        # undoing the old rotation and applying the new one, written as two steps
        undone = oc.rotate_axes(cached, -p_old, axis, base, style)
        assert np.allclose(undone, k_raw, atol=1e-9)
        # scores depend on the per-axis position difference only
        p_q = rng.integers(0, 4000, size=(9, 3))
        shift = np.array([123, -45, 6])
        s0 = np.sum(oc.rotate_axes(q_raw, p_q, axis, base, style) * oc.rotate_axes(k_raw, p_new, axis, base, style), -1)
        s1 = np.sum(oc.rotate_axes(q_raw, p_q + shift, axis, base, style) *
                    oc.rotate_axes(k_raw, p_new + shift, axis, base, style), -1)
        assert np.allclose(s0, s1, atol=1e-8)


def test_axes_rotation_against_transformers_multimodal_helper():
    torch = pytest.importorskip("torch")
    mod = pytest.importorskip("transformers.models.qwen2_vl.modeling_qwen2_vl")
    d, base, n = 32, 1e4, 7
    sections = [4, 6, 6]
    rng = np.random.default_rng(24)
    x = rng.normal(size=(1, 1, n, d))
    pos3 = rng.integers(0, 900, size=(n, 3))
    inv = 1.0 / (base ** (np.arange(0, d, 2, dtype=np.float64) / d))
    ang = pos3.T[:, None, :, None] * inv                  # [3, 1, n, d/2]: every axis at every frequency
    emb = np.concatenate([ang, ang], axis=-1)
    cos, sin = torch.from_numpy(np.cos(emb)), torch.from_numpy(np.sin(emb))
    xt = torch.from_numpy(x)
    want, _ = mod.apply_multimodal_rotary_pos_emb(xt, xt, cos, sin, sections)
    got = oc.rotate_axes(x[0, 0], pos3, _sections_axis_map(sections), base, style=0)
    assert np.allclose(got, want[0, 0].numpy(), atol=1e-12)


def test_rerotate_axes_on_a_pool():
    rng = np.random.default_rng(25)
    n_layers, n_slots, n_heads, d, base = 2, 30, 2, 16, 1e4
    axis = _sections_axis_map([2, 3, 3])
    k = rng.normal(size=(n_layers, n_slots, n_heads, d)).astype(np.float32)
    v = rng.normal(size=(n_layers, n_slots, n_heads, d)).astype(np.float32)
    src, dst = np.array([4, 29, 11], np.int32), np.array([0, 1, 2], np.int32)
    delta3 = np.array([[-256, 0, 0], [3, -2, 7], [0, 0, 0]], np.int32)
    k_rows, v_rows = oc.rerotate_axes(k, v, src, dst, delta3, axis, base)
    for r in range(3):
        for l in range(n_layers):
            want = oc.rotate_axes(k[l, src[r]].astype(np.float64), delta3[r], axis, base)
            assert np.allclose(k_rows[r, l], want, atol=1e-13)
            assert np.array_equal(v_rows[r, l], v[l, src[r]].astype(np.float64))
    assert np.array_equal(k_rows[2], k[:, 11].astype(np.float64))
    # a time-only shift with every pair on the time axis is the one-dimensional correction
    k1, _ = oc.rerotate(k, v, src, dst, delta3[:, 0], base)
    k3, _ = oc.rerotate_axes(k, v, src, dst, delta3 * np.array([1, 0, 0]), np.zeros(d // 2, np.int64), base)
    assert np.allclose(k1, k3, atol=1e-13)


# ------------------------------------------------------------------ (c) scatter
def test_scatter_writes_targets_and_nothing_else():
    rng = np.random.default_rng(20)
    cache = rng.normal(size=(32, 2, 8)).astype(np.float32)
    before = cache.copy()
    new = rng.normal(size=(5, 2, 8)).astype(np.float32)
    slot = np.array([7, -1, 0, 31, 12], np.int32)
    oc.scatter(cache, new, slot)
    for i, s in enumerate(slot):
        if s >= 0:
            assert np.array_equal(cache[s], new[i])
    untouched = np.setdiff1d(np.arange(32), slot[slot >= 0])
    assert np.array_equal(cache[untouched], before[untouched])


# ------------------------------------------------------------------ (d) attention
def _attn_loops(q, k, v, q_pos, scale, rep):
    """Per-element Python loops straight from the definition (tiny inputs only)."""
    n_q, n_heads, d = q.shape
    out = np.zeros((n_q, n_heads, d))
    for t in range(n_q):
        for h in range(n_heads):
            g = h // rep
            scores = []
            for j in range(q_pos[t] + 1):
                scores.append(scale * sum(float(q[t, h, c]) * float(k[j, g, c]) for c in range(d)))
            m = max(scores)
            w = [math.exp(x - m) for x in scores]
            z = sum(w)
            for c in range(d):
                out[t, h, c] = sum(w[j] * float(v[j, g, c]) for j in range(len(w))) / z
    return out


def test_window_attention_against_python_loops():
    rng = np.random.default_rng(30)
    n_ctx, d, n_heads, n_kv = 37, 8, 4, 2
    k = rng.normal(size=(48, n_kv, d))
    v = rng.normal(size=(48, n_kv, d))
    perm_blocks = np.array([[2, 0, 1]], np.int32)                # a shuffled block table
    seq_slots = np.array([perm_blocks[0, j // 16] * 16 + j % 16 for j in range(n_ctx)])
    q_pos = np.array([0, 3, 3, 15, 16, 17, 30, 36], np.int32)
    q = rng.normal(size=(q_pos.size, n_heads, d))
    got = oc.window_attn(q, k, v, np.array([0, q_pos.size], np.int32), q_pos, perm_blocks, n_heads,
                         0.3)
    want = _attn_loops(q, k[seq_slots], v[seq_slots], q_pos, 0.3, n_heads // n_kv)
    assert np.allclose(got, want, atol=1e-12)


def test_all_tokens_as_queries_equals_full_causal_and_library_attention():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(31)
    n, d, n_heads, n_kv = 100, 64, 2, 1
    q = rng.normal(size=(n, n_heads, d))
    k = rng.normal(size=(112, n_kv, d))
    v = rng.normal(size=(112, n_kv, d))
    bt = np.arange(7, dtype=np.int32)[None]
    scale = 1.0 / math.sqrt(d)
    got = oc.window_attn(q, k, v, np.array([0, n], np.int32), np.arange(n, dtype=np.int32), bt,
                         n_heads, scale)
    full = oc.full_causal(q, k[:n], v[:n], scale)
    assert np.allclose(got, full, atol=1e-12)
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(k[:n]).permute(1, 0, 2)[None].repeat_interleave(n_heads // n_kv, dim=1)
    tv = torch.from_numpy(v[:n]).permute(1, 0, 2)[None].repeat_interleave(n_heads // n_kv, dim=1)
    lib = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    assert np.allclose(full, lib[0].permute(1, 0, 2).numpy(), atol=1e-10)
    small = _attn_loops(q[:12, :, :8], k[:12, :, :8], v[:12, :, :8], list(range(12)),
                        scale, n_heads // n_kv)
    assert np.allclose(oc.full_causal(q[:12, :, :8], k[:12, :, :8], v[:12, :, :8], scale), small,
                       atol=1e-12)


def test_attention_invariants():
    rng = np.random.default_rng(32)
    n_slots, d, n_heads, n_kv = 64, 16, 4, 2
    k = rng.normal(size=(n_slots, n_kv, d))
    v = rng.normal(size=(n_slots, n_kv, d))
    bt = np.array([[0, 1, 2, 3]], np.int32)
    q_pos = np.array([0, 5, 20, 50], np.int32)
    q = rng.normal(size=(4, n_heads, d))
    cu = np.array([0, 4], np.int32)
    # constant values come back unchanged (weights sum to one)
    out = oc.window_attn(q, k, np.ones_like(v), cu, q_pos, bt, n_heads, 0.25)
    assert np.allclose(out, 1.0, atol=1e-14)
    out = oc.window_attn(q, k, v, cu, q_pos, bt, n_heads, 0.25)
    # a query at index 0 sees only entry 0
    assert np.allclose(out[0, 0], v[0, 0]) and np.allclose(out[0, 3], v[0, 1])
    # entries beyond the causal frontier do not matter
    k2, v2 = k.copy(), v.copy()
    k2[51:] = 99.0
    v2[51:] = -99.0
    assert np.array_equal(oc.window_attn(q, k2, v2, cu, q_pos, bt, n_heads, 0.25), out)
    # permuting the entries below the frontier of the last query leaves its row unchanged
    perm = rng.permutation(51)
    k3, v3 = k.copy(), v.copy()
    k3[:51] = k[perm]
    v3[:51] = v[perm]
    out3 = oc.window_attn(q, k3, v3, cu, q_pos, bt, n_heads, 0.25)
    assert np.allclose(out3[3], out[3], atol=1e-13)
    # a shuffled block table over shuffled storage is the same sequence
    bt2 = np.array([[3, 1, 0, 2]], np.int32)
    k4, v4 = np.empty_like(k), np.empty_like(v)
    for j in range(n_slots):
        k4[bt2[0, j // 16] * 16 + j % 16] = k[j]
        v4[bt2[0, j // 16] * 16 + j % 16] = v[j]
    assert np.allclose(oc.window_attn(q, k4, v4, cu, q_pos, bt2, n_heads, 0.25), out, atol=1e-14)
    # grouped heads: query heads 0,1 read kv head 0; 2,3 read kv head 1 -> equals MHA on repeated KV
    out_mha = oc.window_attn(q, np.repeat(k, 2, axis=1), np.repeat(v, 2, axis=1), cu, q_pos, bt,
                             n_heads, 0.25)
    assert np.allclose(out_mha, out, atol=1e-14)
    # row subset: evaluating only some queries gives those rows
    sub = oc.window_attn(q, k, v, cu, q_pos, bt, n_heads, 0.25, rows=[1, 3])
    assert np.array_equal(sub, out[[1, 3]])


def test_two_streams_use_their_own_tables():
    rng = np.random.default_rng(33)
    k = rng.normal(size=(64, 1, 8))
    v = rng.normal(size=(64, 1, 8))
    q = rng.normal(size=(5, 2, 8))
    bt = np.array([[1, 3], [2, 0]], np.int32)
    cu = np.array([0, 2, 5], np.int32)
    q_pos = np.array([4, 20, 0, 17, 31], np.int32)
    out = oc.window_attn(q, k, v, cu, q_pos, bt, 2, 0.5)
    for s, rows in ((0, [0, 1]), (1, [2, 3, 4])):
        slots = np.array([bt[s, j // 16] * 16 + j % 16 for j in range(32)])
        want = _attn_loops(q[rows], k[slots], v[slots], q_pos[rows], 0.5, 2)
        assert np.allclose(out[rows], want, atol=1e-12)
