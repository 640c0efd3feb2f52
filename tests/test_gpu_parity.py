"""GPU-vs-oracle parity through the C ABI (needs an MI355X: `-m gpu`).

Integer / byte / index results must match bit for bit; re-rotated keys within 1e-2 max-abs and
attention within 2e-2 max-abs, 1e-2 mean-relative of the float64 oracle (see tests/helpers.py).
Every case prints what it is about to run before touching the GPU.
"""
import math
import sys

import numpy as np
import pytest
import torch

from oracle import codecsight_oracle as oc
from paper_2604_06036_amd import engine, planner, synth
from tests import helpers as hp

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def cs():
    from paper_2604_06036_amd import binding
    say(f"library: {binding.cs_version()} on {torch.cuda.get_device_name(0)}")
    return binding


# =============================================================================== (a) scoring
def _score_gpu(cs, mv, sad, intra, ft, cu, acc, gh, gw, g, tmv, tsad, use_res):
    n_frames, n_streams = int(ft.shape[0]), int(cu.shape[0]) - 1
    t_per = (gh // g) * (gw // g)
    d = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    d_acc = d(acc)
    keep = torch.full((max(1, n_frames), t_per), 9, dtype=torch.uint8, device=DEV)
    idx = torch.full((max(1, n_frames * t_per),), -7, dtype=torch.int32, device=DEV)
    off = torch.full((n_frames + 1,), -7, dtype=torch.int32, device=DEV)
    nbytes = cs.cs_score_compact_workspace(n_streams, n_frames, gh, gw, g)
    ws = torch.randint(0, 255, (max(8, nbytes),), dtype=torch.uint8, device=DEV)   # dirty workspace
    cs.cs_score_compact(d(mv), d(None if sad is None else sad.view(np.int32)), d(intra), d(ft), d(cu),
                        d_acc, n_streams, n_frames, gh, gw, g, tmv, tsad, use_res, keep, idx, off, ws, nbytes)
    torch.cuda.synchronize()
    if n_streams > 0 and n_frames > 0:
        assert int(ws[4:8].view(torch.int32).item()) == 0, "look-back wait ran into its bound"
    return (keep.cpu().numpy()[:n_frames], idx.cpu().numpy(), off.cpu().numpy(),
            None if d_acc is None else d_acc.cpu().numpy())


def _score_case(cs, rng, n_streams, frames_per_stream, gh, gw, g, tmv, tsad, use_res, with_acc,
                with_intra, p_iframe=0.15, spread=12):
    counts = np.asarray(frames_per_stream, np.int32)
    cu = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    n_frames, n_patch = int(cu[-1]), gh * gw
    mv = np.rint(rng.normal(0, spread, size=(n_frames, n_patch, 2))).astype(np.int16)
    sad = rng.integers(0, 1200, size=(n_frames, n_patch), dtype=np.uint32)
    ft = (rng.random(n_frames) < p_iframe).astype(np.uint8)
    intra = (rng.random((n_frames, n_patch)) < 0.02).astype(np.uint8) * 3 if with_intra else None
    acc = (rng.random((n_streams, n_patch)) < 0.1).astype(np.uint8) if with_acc else None
    want = oc.score_compact(mv, sad if use_res else None, intra, ft, cu, acc, gh, gw, g, tmv, tsad, use_res)
    got = _score_gpu(cs, mv, sad if use_res else None, intra, ft, cu, acc, gh, gw, g, tmv, tsad, use_res)
    keep_w, idx_w, off_w, acc_w = want
    keep_g, idx_g, off_g, acc_g = got
    assert np.array_equal(keep_g, keep_w)
    assert np.array_equal(off_g, off_w)
    assert np.array_equal(idx_g[: idx_w.size], idx_w)
    assert np.all(idx_g[idx_w.size:] == -7)                      # the tail is left untouched
    if with_acc:
        assert np.array_equal(acc_g != 0, acc_w != 0)
    return int(idx_w.size)


SCORE_CASES = [
    # streams, frames per stream,            grid,     g, tmv, tsad, res,  acc,  intra
    (1, [1], (16, 16), 1, 17, 401, True, True, False),
    (1, [4], (16, 16), 1, 17, 401, True, False, False),
    (3, [2, 0, 5], (16, 16), 1, 100, 600, True, True, True),       # a stream with no frames
    (5, [1, 1, 1, 1, 1], (26, 46), 1, 150, 900, True, True, False),  # T = 1196: ragged sweeps
    (9, [3] * 9, (7, 9), 1, 60, 500, False, True, True),           # T = 63 < one wave
    (4, [2, 3, 1, 2], (32, 32), 2, 200, 800, True, True, True),     # 2x2 projection groups
    (2, [2, 2], (6, 10), 2, 90, 300, True, False, False),
    (37, [1] * 37, (16, 16), 1, 300, 1000, True, True, False),     # 10 tiles of 4 streams
    (301, list(np.random.default_rng(5).integers(0, 4, 301)), (8, 8), 1, 250, 900, True, True, False),
    (2, [40, 3], (16, 16), 1, 120, 700, True, True, False),          # > 128 ballot words in one wave
    (2, [3, 3], (16, 16), 1, 0, 0, True, True, False),              # zero thresholds: keep all
    (2, [3, 3], (16, 16), 1, 0xFFFFFFFF, 0xFFFFFFFF, True, False, False),   # nothing kept
]


@pytest.mark.parametrize("case", range(len(SCORE_CASES)))
def test_score_compact_random(cs, case):
    n_streams, fps, (gh, gw), g, tmv, tsad, res, acc, intra = SCORE_CASES[case]
    say(f"score_compact case {case}: streams={n_streams} frames={sum(fps)} grid={gh}x{gw} g={g} "
        f"tau=({tmv},{tsad}) res={res} acc={acc} intra={intra}")
    rng = np.random.default_rng(1000 + case)
    p_i = 0.0 if tmv == 0xFFFFFFFF else 0.15
    kept = _score_case(cs, rng, n_streams, fps, gh, gw, g, tmv, tsad, res, acc, intra, p_iframe=p_i)
    if tmv == 0:
        assert kept == sum(fps) * (gh // g) * (gw // g)
    if tmv == 0xFFFFFFFF:
        assert kept == 0


def test_score_compact_empty_batch(cs):
    say("score_compact: zero frames / zero streams")
    off = torch.full((1,), -5, dtype=torch.int32, device=DEV)
    cs.cs_score_compact(None, None, None, None, None, None, 0, 0, 16, 16, 1, 17, 401, False, None, None,
                        off, None, 0)
    torch.cuda.synchronize()
    assert off.cpu().tolist() == [0]


def test_score_compact_many_tiles(cs):
    # 4096 streams x 1 frame x 256 tokens: 1024 tiles chained by the look-back
    say("score_compact: 4096 streams, 1024 look-back tiles")
    rng = np.random.default_rng(77)
    _score_case(cs, rng, 4096, [1] * 4096, 16, 16, 1, 400, 1100, True, True, False, p_iframe=0.1)


def test_score_compact_waves_sweeping_several_streams(cs):
    # above 8192 streams a wave sweeps several consecutive streams (here 3 per wave, ragged tail)
    say("score_compact: 20011 streams with 0..2 frames each")
    rng = np.random.default_rng(78)
    _score_case(cs, rng, 20011, list(rng.integers(0, 3, 20011)), 8, 8, 1, 300, 1000, True, True, False)


@pytest.mark.parametrize("n_streams,grid,group,max_frames", [
    (4097, (16, 16), 1, 2),        # just past the one-launch limit, packed lanes
    (5003, (4, 6), 2, 3),          # token groups of 2 x 2 patches
    (6001, (3, 5), 1, 2),          # patch count not a multiple of 4: one location per lane and group
    (4100, (20, 20), 1, 3),        # 400 token locations: two sweeps per frame
])
def test_score_compact_three_launch_form(cs, n_streams, grid, group, max_frames):
    """Batches above 4096 streams run as score / scan / emit launches: every variant of the kernel
    body in that form, ragged frame counts (streams without frames included)."""
    say(f"score_compact three-launch form: {n_streams} streams, grid {grid}, group {group}")
    rng = np.random.default_rng(90 + n_streams)
    _score_case(cs, rng, n_streams, list(rng.integers(0, max_frames + 1, n_streams)), grid[0], grid[1], group,
                200, 900, True, True, True)


def test_score_compact_i_frame_ignores_metadata(cs):
    say("score_compact: garbage in I-frame metadata")
    rng = np.random.default_rng(3)
    n_patch = 256
    ft = np.array([1, 0, 1, 0], np.uint8)
    cu = np.array([0, 2, 4], np.int32)
    mv = np.rint(rng.normal(0, 3, size=(4, n_patch, 2))).astype(np.int16)
    sad = rng.integers(0, 500, size=(4, n_patch), dtype=np.uint32)
    acc = np.ones((2, n_patch), np.uint8)
    a = _score_gpu(cs, mv, sad, None, ft, cu, acc, 16, 16, 1, 17, 401, True)
    mv[[0, 2]] = 32767
    sad[[0, 2]] = 0xFFFFFFFF
    b = _score_gpu(cs, mv, sad, None, ft, cu, acc, 16, 16, 1, 17, 401, True)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    assert a[0][0].all() and a[0][2].all()


# =============================================================================== (m) projection
def _project_gpu(cs, blocks, cu, geom):
    n_frames = len(cu) - 1
    gh, gw = geom[5], geom[6]
    raw = torch.from_numpy(np.ascontiguousarray(blocks).view(np.uint8).copy()) if blocks.size else torch.zeros(16, dtype=torch.uint8)
    d_blocks = raw.to(DEV)
    d_cu = torch.from_numpy(np.asarray(cu, np.int32)).to(DEV)
    mv = torch.full((max(1, n_frames), gh * gw, 2), -99, dtype=torch.int16, device=DEV)
    intra = torch.full((max(1, n_frames), gh * gw), 77, dtype=torch.uint8, device=DEV)
    cs.cs_project_blocks(d_blocks, d_cu, n_frames, geom[0], geom[1], geom[2], geom[3], geom[4], gh, gw, mv, intra,
                         n_blocks=int(blocks.size))
    torch.cuda.synchronize()
    return mv.cpu().numpy()[:n_frames], intra.cpu().numpy()[:n_frames]


def _random_block_frames(rng, counts, src_w, src_h, max_size, spread, p_intra=0.1, extremes=False):
    from oracle import projection_oracle as po
    n = int(sum(counts))
    b = np.zeros(n, po.BLOCK_DTYPE)
    b["x"] = rng.integers(0, src_w + 3, size=n)                 # some start outside the frame
    b["y"] = rng.integers(0, src_h + 3, size=n)
    b["w"] = rng.integers(0, max_size + 1, size=n)              # some have no area
    b["h"] = rng.integers(0, max_size + 1, size=n)
    b["dx"] = rng.integers(-spread, spread + 1, size=n)
    b["dy"] = rng.integers(-spread, spread + 1, size=n)
    b["flags"] = (rng.random(n) < p_intra).astype(np.uint32) | (rng.integers(0, 4, size=n).astype(np.uint32) << 1)
    if extremes and n >= 4:
        b["dx"][:4], b["dy"][:4] = (-32768, 32767, -32768, 0), (-32768, 32767, 32767, -32768)
        b["flags"][:4] = 0
        b["w"][:4], b["h"][:4] = max(1, max_size), max(1, max_size)
    cu = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    return b, cu


PROJECT_CASES = [
    # src_w, src_h, in_w, in_h, patch, gh, gw | blocks per frame | max block | vector spread | extremes
    ((64, 48, 32, 24, 8, 3, 4), [7, 0, 30], 20, 9, False),
    ((30, 10, 20, 10, 5, 2, 4), [12, 12], 8, 3, False),
    ((1920, 1080, 448, 448, 28, 16, 16), [3000, 1, 5000], 64, 40, True),
    ((1920, 1088, 1288, 728, 28, 26, 46), [9000], 32, 30, False),
    ((17, 23, 12, 18, 3, 6, 4), [40] * 5, 12, 2, False),                  # many ties
    ((13, 9, 26, 27, 9, 3, 3), [25], 6, 5, False),                        # upscaling
    ((31, 19, 14, 14, 7, 1, 1), [25], 31, 5, False),                      # grid smaller than the input
    ((16384, 16384, 16384, 16384, 1024, 16, 16), [500], 5000, 32767, True),   # the largest numerators
    ((4000, 3000, 7168, 14, 14, 1, 512), [2000], 300, 100, False),
    ((640, 360, 1792, 56, 14, 4, 128), [4000, 4000], 40, 100, True),
    ((1, 1, 1, 1, 1, 1, 1), [3], 1, 3, False),
]


@pytest.mark.parametrize("case", range(len(PROJECT_CASES)))
def test_project_blocks(cs, case):
    """Projected vectors and intra flags equal the oracle's bit for bit (the tie rule makes the
    result unique), on awkward scalings, clipped and empty footprints and extreme vectors."""
    from oracle import projection_oracle as po
    geom, counts, max_size, spread, extremes = PROJECT_CASES[case]
    say(f"project_blocks case {case}: geometry {geom} blocks {counts}")
    rng = np.random.default_rng(8000 + case)
    blocks, cu = _random_block_frames(rng, counts, geom[0], geom[1], max_size, spread, extremes=extremes)
    mv_w, intra_w = po.project_blocks(blocks, cu, *geom)
    mv_g, intra_g = _project_gpu(cs, blocks, cu, geom)
    assert np.array_equal(mv_g, mv_w) and np.array_equal(intra_g, intra_w)
    # block order inside a frame does not matter
    perm = np.concatenate([cu[f] + rng.permutation(cu[f + 1] - cu[f]) for f in range(len(cu) - 1)]).astype(np.int64)
    mv_p, intra_p = _project_gpu(cs, blocks[perm], cu, geom)
    assert np.array_equal(mv_p, mv_w) and np.array_equal(intra_p, intra_w)


def test_project_blocks_no_frames(cs):
    say("project_blocks with no frames")
    from oracle import projection_oracle as po
    mv, intra = _project_gpu(cs, np.zeros(0, po.BLOCK_DTYPE), np.zeros(1, np.int32), (64, 48, 32, 24, 8, 3, 4))
    assert mv.shape[0] == 0 and intra.shape[0] == 0


@pytest.mark.parametrize("w", [synth.small_variant(synth.CFG2, n_streams=3), synth.CFG3P], ids=lambda w: w.name)
def test_projection_feeds_scoring(cs, w):
    """Decoder-shaped block lists (macroblock partitions of a 1920x1080 frame) -> projection ->
    scoring, HIP chain against oracle chain: the projected metadata and the kept-token lists agree."""
    from oracle import projection_oracle as po
    say(f"projection -> scoring: {w.name}")
    src_w, src_h = synth.SOURCE_SIZE
    in_w, in_h = synth.input_size(w)
    geom = (src_w, src_h, in_w, in_h, synth.MODEL_PATCH, w.grid_h, w.grid_w)
    ftypes, blobs = [], []
    for s in range(w.n_streams):
        m = synth.stream_metadata(w, s)
        ftypes.append(m.frame_type[-w.stride:])
        blobs.append(m.blob[-w.stride:])
    ftype = np.concatenate(ftypes)
    blocks, cu = synth.block_frames(w, ftype, np.concatenate(blobs))
    say(f"  {blocks.size} blocks in {ftype.size} frames")
    mv_w, intra_w = po.project_blocks(blocks.view(po.BLOCK_DTYPE), cu, *geom)
    mv_g, intra_g = _project_gpu(cs, blocks, cu, geom)
    assert np.array_equal(mv_g, mv_w) and np.array_equal(intra_g, intra_w)
    cu_frames = (np.arange(w.n_streams + 1) * w.stride).astype(np.int32)
    acc = np.zeros((w.n_streams, w.patches), np.uint8)
    want = oc.score_compact(mv_w, None, intra_w, ftype, cu_frames, acc.copy(), w.grid_h, w.grid_w, w.group,
                            w.tau_mv_sq, 0, False)
    got = _score_gpu(cs, mv_g, None, intra_g, ftype, cu_frames, acc.copy(), w.grid_h, w.grid_w, w.group,
                     w.tau_mv_sq, 0, False)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[2], want[2])
    assert np.array_equal(got[1][: want[1].size], want[1])
    say(f"  kept {want[1].size} of {ftype.size * w.tokens_per_frame} tokens")


# =============================================================================== (r) residual proxy
def _residual_gpu(cs, cur, prev, field, cell, in_w, in_h, patch, gh, gw, pad=0):
    """cur, prev: uint8 [F, H, W] on the host; rows are copied into planes with pitch = W rounded
    up to 16 (+ pad) whose padding bytes hold garbage, so a read past a row's end would show."""
    n_frames, h, w = cur.shape
    pitch = -(-w // 16) * 16 + pad
    def plane(a, fill):
        t = np.full((max(1, n_frames), h, pitch), fill, np.uint8)
        t[:n_frames, :, :w] = a
        return torch.from_numpy(t).to(DEV)
    d_cur, d_prev = plane(cur, 201), plane(prev, 57)
    d_field = torch.from_numpy(np.ascontiguousarray(field)).to(DEV) if field.size else torch.zeros(2, dtype=torch.int16, device=DEV)
    res = torch.full((max(1, n_frames), gh * gw), 12345, dtype=torch.int32, device=DEV)
    cs.cs_residual_proxy(d_cur, d_prev, d_field, n_frames, w, h, pitch, h * pitch, cell, in_w, in_h, patch, gh, gw, res)
    torch.cuda.synchronize()
    return res.cpu().numpy().view(np.uint32)[:n_frames]


RESIDUAL_CASES = [
    # frames, h, w, cell, in_w, in_h, patch, gh, gw, vector spread (quarter pixels), pad
    (1, 4, 8, 4, 4, 2, 2, 1, 2, 8, 0),
    (2, 12, 20, 4, 15, 9, 3, 3, 5, 40, 0),
    (3, 10, 30, 4, 20, 10, 5, 2, 4, 60, 16),
    (1, 37, 53, 8, 26, 27, 9, 3, 2, 200, 0),            # width and height not multiples of the cell
    (2, 64, 200, 16, 100, 32, 8, 4, 12, 100, 32),
    (1, 18, 31, 16, 14, 14, 7, 1, 1, 30, 0),            # grid smaller than the input
    (2, 40, 300, 4, 140, 56, 28, 2, 5, 2000, 0),        # vectors far beyond the frame: clamped references
    (1, 270, 480, 4, 112, 112, 7, 16, 16, 90, 0),
    (1, 90, 4200, 8, 1288, 28, 28, 1, 46, 300, 0),      # more than 256 chunks per row
    (5, 30, 64, 4, 64, 32, 4, 8, 16, 24, 0),            # patch columns exactly four pixels wide
]


@pytest.mark.parametrize("case", range(len(RESIDUAL_CASES)))
def test_residual_proxy(cs, case):
    """Per-patch residual scores equal the oracle's bit for bit (integer sums, exact division)."""
    from oracle import residual_oracle as ro
    n_frames, h, w, cell, in_w, in_h, patch, gh, gw, spread, pad = RESIDUAL_CASES[case]
    say(f"residual_proxy case {case}: {n_frames} frames {w}x{h} cell {cell} -> grid {gh}x{gw}")
    rng = np.random.default_rng(9000 + case)
    cur = rng.integers(0, 256, size=(n_frames, h, w), dtype=np.uint8)
    prev = rng.integers(0, 256, size=(n_frames, h, w), dtype=np.uint8)
    field = rng.integers(-spread, spread + 1, size=(n_frames, -(-h // cell), -(-w // cell), 2)).astype(np.int16)
    field[:, 0, 0] = (32767, -32768)
    want = ro.residual_proxy(cur, prev, field, cell, in_w, in_h, patch, gh, gw)
    got = _residual_gpu(cs, cur, prev, field, cell, in_w, in_h, patch, gh, gw, pad)
    assert np.array_equal(got, want)


def test_residual_proxy_closed_forms_on_gpu(cs):
    """Exact translation scores 0 everywhere; a constant offset k scores 256 k; no frames is fine."""
    say("residual_proxy closed forms")
    rng = np.random.default_rng(9100)
    h, w = 48, 96
    prev = rng.integers(0, 200, size=(1, h, w), dtype=np.uint8)
    ys, xs = np.meshgrid(np.arange(h), np.arange(w), indexing="ij")
    cur = prev[:, np.clip(ys - 2, 0, h - 1), np.clip(xs + 3, 0, w - 1)]
    field = np.zeros((1, h // 4, w // 4, 2), np.int16)
    field[..., 0], field[..., 1] = 12, -8
    assert not _residual_gpu(cs, cur, prev, field, 4, 48, 24, 8, 3, 6).any()
    field[:] = 0
    assert np.all(_residual_gpu(cs, prev + 9, prev, field, 4, 48, 24, 8, 3, 6) == 256 * 9)
    assert _residual_gpu(cs, cur[:0], prev[:0], field[:0], 4, 48, 24, 8, 3, 6).shape == (0, 18)


def test_residual_proxy_feeds_rescue(cs):
    """Decoder-shaped inputs (1920x1080 planes, macroblock partitions) -> projection + residual
    proxy -> scoring with residual rescue on, HIP chain against oracle chain."""
    from oracle import projection_oracle as po
    from oracle import residual_oracle as ro
    w = synth.small_variant(synth.CFG2, n_streams=2)
    say(f"projection + residual proxy -> scoring: {w.name}")
    src_w, src_h = synth.SOURCE_SIZE
    in_w, in_h = synth.input_size(w)
    metas = [synth.stream_metadata(w, s) for s in range(w.n_streams)]
    ftype = np.concatenate([m.frame_type[-w.stride:] for m in metas])
    blob = np.concatenate([m.blob[-w.stride:] for m in metas])
    ftype[:] = 0                                              # P-frames, so that the metadata decides
    blocks, cu = synth.block_frames(w, ftype, blob)
    field = synth.motion_field(blocks, cu, 4)
    cur, prev = synth.decoded_frames(w, ftype.size, blob)
    geom = (src_w, src_h, in_w, in_h, synth.MODEL_PATCH, w.grid_h, w.grid_w)
    mv_w, intra_w = po.project_blocks(blocks.view(po.BLOCK_DTYPE), cu, *geom)
    res_w = ro.residual_proxy(cur, prev, field, 4, in_w, in_h, synth.MODEL_PATCH, w.grid_h, w.grid_w)
    mv_g, intra_g = _project_gpu(cs, blocks, cu, geom)
    res_g = _residual_gpu(cs, cur, prev, field, 4, in_w, in_h, synth.MODEL_PATCH, w.grid_h, w.grid_w)
    assert np.array_equal(res_g, res_w) and np.array_equal(mv_g, mv_w)
    tau_res = int(0.05 * 255 * 256)                           # 5 % of full scale, in 1/256 grey levels
    cu_frames = (np.arange(w.n_streams + 1) * w.stride).astype(np.int32)
    acc = np.zeros((w.n_streams, w.patches), np.uint8)
    want = oc.score_compact(mv_w, res_w, intra_w, ftype, cu_frames, acc.copy(), w.grid_h, w.grid_w, w.group,
                            w.tau_mv_sq, tau_res, True)
    got = _score_gpu(cs, mv_g, res_g, intra_g, ftype, cu_frames, acc.copy(), w.grid_h, w.grid_w, w.group,
                     w.tau_mv_sq, tau_res, True)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[2], want[2])
    no_rescue = oc.score_compact(mv_w, None, intra_w, ftype, cu_frames, acc.copy(), w.grid_h, w.grid_w, w.group,
                                 w.tau_mv_sq, 0, False)
    say(f"  kept {want[1].size} tokens with rescue, {no_rescue[1].size} without, of {ftype.size * w.tokens_per_frame}")
    assert want[1].size > no_rescue[1].size


# =============================================================================== (b) re-rotation
def _pool(rng, shape, dtype):
    x = torch.from_numpy(rng.normal(size=shape).astype(np.float32))
    return x if dtype == "f32" else x.to(torch.bfloat16)


REROT_CASES = [
    # dtype, L, n_slots, Hkv, d, n_rows, style, repack, base, layout
    ("f32", 1, 512, 1, 64, 120, 0, True, 1e4, "lshd"),
    ("f32", 3, 256, 2, 128, 77, 1, False, 1e6, "lshd"),
    ("bf16", 28, 1024, 4, 128, 490, 0, True, 1e6, "lshd"),
    ("bf16", 5, 640, 8, 128, 333, 0, False, 1e6, "lshd"),
    ("bf16", 2, 640, 3, 64, 200, 1, True, 1e4, "lshd"),
    ("bf16", 7, 640, 4, 128, 250, 0, True, 1e6, "lhsd"),       # head-major pool: stride_head != d
    ("bf16", 9, 300, 2, 256, 100, 0, True, 5e5, "lshd"),
    ("bf16", 1, 64, 1, 16, 1, 0, True, 1e4, "lshd"),
]


@pytest.mark.parametrize("case", range(len(REROT_CASES)))
def test_kv_rerotate(cs, case):
    dtype, n_layers, n_slots, n_heads, d, n_rows, style, repack, base, layout = REROT_CASES[case]
    say(f"kv_rerotate case {case}: {dtype} L={n_layers} slots={n_slots} Hkv={n_heads} d={d} rows={n_rows} "
        f"style={style} repack={repack} layout={layout}")
    rng = np.random.default_rng(2000 + case)
    if layout == "lshd":
        k = _pool(rng, (n_layers, n_slots, n_heads, d), dtype)
        v = _pool(rng, (n_layers, n_slots, n_heads, d), dtype)
        view = lambda t: t
    else:
        k = _pool(rng, (n_layers, n_heads, n_slots, d), dtype)
        v = _pool(rng, (n_layers, n_heads, n_slots, d), dtype)
        view = lambda t: t.permute(0, 2, 1, 3)                  # logical [L, slot, head, d]
    assert (2 if repack else 1) * n_rows <= n_slots, "case needs disjoint source and destination slots"
    perm = rng.permutation(n_slots)
    src = perm[:n_rows].astype(np.int32)
    dst = perm[n_rows: 2 * n_rows].astype(np.int32) if repack else None
    delta = rng.integers(-2392, 2393, size=n_rows).astype(np.int32)
    delta[: min(3, n_rows)] = [0, -256, 2392][: min(3, n_rows)]

    k_ref, v_ref = oc.rerotate(hp.f64(view(k)), hp.f64(view(v)), src, dst, delta, base, style)

    kd, vd = k.to(DEV), v.to(DEV)
    kv_, vv_ = view(kd), view(vd)
    cs.cs_kv_rerotate(kd, vd if repack else None, torch.from_numpy(src).to(DEV),
                      torch.from_numpy(dst).to(DEV) if repack else None, torch.from_numpy(delta).to(DEV),
                      n_rows, n_layers, n_heads, d, kv_.stride(0), kv_.stride(1), kv_.stride(2), base, style,
                      cs.CS_BF16 if dtype == "bf16" else cs.CS_F32)
    torch.cuda.synchronize()
    k_out, v_out = view(kd.cpu()), view(vd.cpu())
    tgt = dst if repack else src
    got_rows = k_out[:, torch.from_numpy(tgt.astype(np.int64))].permute(1, 0, 2, 3).contiguous()
    stats = hp.check_rerotated(got_rows, k_ref, dtype)
    say(f"  -> {stats}")
    if repack:                                                   # values copied bit for bit
        assert torch.equal(v_out[:, torch.from_numpy(dst.astype(np.int64))],
                           view(v)[:, torch.from_numpy(src.astype(np.int64))])
    # every other row of the pool is bit-unchanged
    other = np.setdiff1d(np.arange(n_slots), tgt)
    oi = torch.from_numpy(other)
    assert torch.equal(k_out[:, oi], view(k)[:, oi]) and torch.equal(v_out[:, oi], view(v)[:, oi])
    if not repack:
        assert torch.equal(v_out, view(v))


def test_kv_rerotate_closed_form_on_gpu(cs):
    """Keys cached at p_old, corrected by delta, equal keys computed at p_old + delta (Eq. 6)."""
    say("kv_rerotate: closed form R(delta) R(p) k == R(p + delta) k, fp32 storage")
    rng = np.random.default_rng(42)
    n, d, base = 300, 128, 1e6
    k_raw = rng.normal(size=(n, d))
    p_old = rng.integers(0, 20001, size=n)
    delta = rng.integers(-2392, 2393, size=n).astype(np.int32)
    cached = torch.from_numpy(oc.rotate(k_raw, p_old, base).astype(np.float32)).reshape(1, n, 1, d).to(DEV)
    cs.cs_kv_rerotate(cached, None, torch.arange(n, dtype=torch.int32, device=DEV), None,
                      torch.from_numpy(delta).to(DEV), n, 1, 1, d, n * d, d, d, base, 0, cs.CS_F32)
    torch.cuda.synchronize()
    want = oc.rotate(k_raw, p_old + delta, base)
    assert np.abs(hp.f64(cached.reshape(n, d)) - want).max() <= 2e-5


# ------------------------------------------------------------------ (b') multi-axis correction
def _sections_axis_map(sections, half, interleave=False):
    """Frequency pairs -> axis: consecutive sections (Qwen2-VL style) or t/h/w interleaved."""
    if interleave:
        return (np.arange(half) % 3).astype(np.uint8)
    m = np.concatenate([np.full(n, a, np.uint8) for a, n in enumerate(sections)])
    assert m.size == half
    return m


AXES_CASES = [
    # dtype, L, n_slots, Hkv, d, n_rows, style, repack, base, sections / interleave
    ("f32", 2, 300, 2, 128, 97, 0, True, 1e6, [16, 24, 24]),
    ("bf16", 28, 1024, 4, 128, 490, 0, True, 1e6, [16, 24, 24]),    # Qwen2-VL's sections, all layers
    ("bf16", 5, 640, 8, 128, 333, 0, False, 1e6, "interleave"),      # axes interleaved over the pairs
    ("bf16", 3, 400, 2, 64, 150, 1, True, 1e4, [8, 12, 12]),         # interleaved element pairs
    ("bf16", 1, 64, 1, 16, 1, 0, True, 1e4, [2, 3, 3]),
]


@pytest.mark.parametrize("case", range(len(AXES_CASES)))
def test_kv_rerotate_axes(cs, case):
    dtype, n_layers, n_slots, n_heads, d, n_rows, style, repack, base, sec = AXES_CASES[case]
    say(f"kv_rerotate_axes case {case}: {dtype} L={n_layers} slots={n_slots} Hkv={n_heads} d={d} rows={n_rows} "
        f"style={style} repack={repack} axes={sec}")
    rng = np.random.default_rng(2500 + case)
    axis = _sections_axis_map(sec, d // 2, interleave=(sec == "interleave"))
    k = _pool(rng, (n_layers, n_slots, n_heads, d), dtype)
    v = _pool(rng, (n_layers, n_slots, n_heads, d), dtype)
    perm = rng.permutation(n_slots)
    src = perm[:n_rows].astype(np.int32)
    dst = perm[n_rows: 2 * n_rows].astype(np.int32) if repack else None
    delta3 = np.stack([rng.integers(-2392, 2393, size=n_rows), rng.integers(-40, 41, size=n_rows),
                       rng.integers(-40, 41, size=n_rows)], axis=1).astype(np.int32)
    delta3[0] = [-256, 0, 0]                                     # the sliding window's own case: time only
    k_ref, _ = oc.rerotate_axes(hp.f64(k), hp.f64(v), src, dst, delta3, axis, base, style)
    kd, vd = k.to(DEV), v.to(DEV)
    cs.cs_kv_rerotate_axes(kd, vd if repack else None, torch.from_numpy(src).to(DEV),
                           torch.from_numpy(dst).to(DEV) if repack else None, torch.from_numpy(delta3).to(DEV),
                           torch.from_numpy(axis).to(DEV), n_rows, n_layers, n_heads, d, kd.stride(0), kd.stride(1),
                           kd.stride(2), base, style, cs.CS_BF16 if dtype == "bf16" else cs.CS_F32)
    torch.cuda.synchronize()
    k_out, v_out = kd.cpu(), vd.cpu()
    tgt = dst if repack else src
    got_rows = k_out[:, torch.from_numpy(tgt.astype(np.int64))].permute(1, 0, 2, 3).contiguous()
    say(f"  -> {hp.check_rerotated(got_rows, k_ref, dtype)}")
    if repack:
        assert torch.equal(v_out[:, torch.from_numpy(dst.astype(np.int64))], v[:, torch.from_numpy(src.astype(np.int64))])
    other = torch.from_numpy(np.setdiff1d(np.arange(n_slots), tgt))
    assert torch.equal(k_out[:, other], k[:, other]) and torch.equal(v_out[:, other], v[:, other])
    # row 0 shifted in time only: the pairs of the other two axes come back bit for bit
    ia = np.arange(d // 2) if style == 0 else 2 * np.arange(d // 2)
    ib = ia + d // 2 if style == 0 else ia + 1
    still = torch.from_numpy(np.concatenate([ia[axis != 0], ib[axis != 0]]))
    assert torch.equal(k_out[:, int(tgt[0])][..., still], k[:, int(src[0])][..., still])


def test_kv_rerotate_axes_with_one_axis_equals_plain_call(cs):
    say("kv_rerotate_axes: every pair on the time axis == cs_kv_rerotate, bit for bit")
    rng = np.random.default_rng(77)
    n_layers, n_slots, n_heads, d, n_rows = 4, 512, 4, 128, 200
    k = _pool(rng, (n_layers, n_slots, n_heads, d), "bf16")
    src = torch.from_numpy(rng.permutation(n_slots)[:n_rows].astype(np.int32)).to(DEV)
    delta = rng.integers(-2392, 2393, size=n_rows).astype(np.int32)
    delta3 = np.stack([delta, rng.integers(-9, 9, size=n_rows), rng.integers(-9, 9, size=n_rows)], 1).astype(np.int32)
    a, b = k.to(DEV), k.to(DEV)
    cs.cs_kv_rerotate(a, None, src, None, torch.from_numpy(delta).to(DEV), n_rows, n_layers, n_heads, d,
                      a.stride(0), a.stride(1), a.stride(2), 1e6, 0, cs.CS_BF16)
    cs.cs_kv_rerotate_axes(b, None, src, None, torch.from_numpy(delta3).to(DEV),
                           torch.zeros(d // 2, dtype=torch.uint8, device=DEV), n_rows, n_layers, n_heads, d,
                           b.stride(0), b.stride(1), b.stride(2), 1e6, 0, cs.CS_BF16)
    torch.cuda.synchronize()
    assert torch.equal(a.cpu(), b.cpu())


# =============================================================================== (c) scatter
@pytest.mark.parametrize("dtype,n_tok,n_heads,d,layout", [
    ("f32", 332, 1, 64, "shd"), ("bf16", 425, 4, 128, "shd"), ("bf16", 1000, 8, 128, "hsd"),
    ("bf16", 1, 2, 64, "shd"), ("f32", 63, 3, 128, "shd")])
def test_kv_refresh_scatter(cs, dtype, n_tok, n_heads, d, layout):
    say(f"kv_refresh_scatter: {dtype} tokens={n_tok} Hkv={n_heads} d={d} layout={layout}")
    rng = np.random.default_rng(n_tok * 7 + d)
    n_slots = 2 * n_tok + 40
    shape = (n_slots, n_heads, d) if layout == "shd" else (n_heads, n_slots, d)
    view = (lambda t: t) if layout == "shd" else (lambda t: t.permute(1, 0, 2))
    kc, vc = _pool(rng, shape, dtype), _pool(rng, shape, dtype)
    kn, vn = _pool(rng, (n_tok, n_heads, d), dtype), _pool(rng, (n_tok, n_heads, d), dtype)
    slot = rng.permutation(n_slots)[:n_tok].astype(np.int32)
    slot[rng.random(n_tok) < 0.1] = -1
    raw = torch.int16 if dtype == "bf16" else torch.int32
    k_want = view(kc).contiguous().view(raw).numpy().copy()
    v_want = view(vc).contiguous().view(raw).numpy().copy()
    oc.scatter(k_want, kn.view(raw).numpy(), slot)
    oc.scatter(v_want, vn.view(raw).numpy(), slot)
    kd, vd = kc.to(DEV), vc.to(DEV)
    cs.cs_kv_refresh_scatter(kn.to(DEV), vn.to(DEV), torch.from_numpy(slot).to(DEV), kd, vd, n_tok, n_heads,
                             d, view(kd).stride(0), view(kd).stride(1),
                             cs.CS_BF16 if dtype == "bf16" else cs.CS_F32)
    torch.cuda.synchronize()
    assert np.array_equal(view(kd.cpu()).contiguous().view(raw).numpy(), k_want)
    assert np.array_equal(view(vd.cpu()).contiguous().view(raw).numpy(), v_want)


# =============================================================================== (d) attention
def _attn_case(cs, rng, dtype, n_q_heads, n_kv_heads, d, kv_lens, n_qs, shuffle=True, poison=True,
               all_queries=False, scale_mult=1.0, late_outlier=0.0):
    """`scale_mult` multiplies the softmax scale (peaked rows: the running maximum keeps rising along
    the sweep); `late_outlier` > 0 multiplies one key row near the end of every stream by that
    factor (a maximum that jumps late, past the first tile and past the first key range of a split
    sweep)."""
    n_streams = len(kv_lens)
    nb = [(-(-L // 16)) for L in kv_lens]
    max_blocks = max(nb) + 1
    n_blocks = sum(nb) + 3
    ids = rng.permutation(n_blocks) if shuffle else np.arange(n_blocks)
    bt = np.full((n_streams, max_blocks), 0, np.int32)
    at = 0
    for s in range(n_streams):
        bt[s, : nb[s]] = ids[at: at + nb[s]]
        at += nb[s]
    kc = _pool(rng, (n_blocks * 16, n_kv_heads, d), dtype)
    vc = _pool(rng, (n_blocks * 16, n_kv_heads, d), dtype)
    q_pos, cu = [], [0]
    for s in range(n_streams):
        if all_queries:
            pos = np.arange(kv_lens[s])
        else:
            pos = np.sort(rng.choice(kv_lens[s], size=n_qs[s], replace=False)) if n_qs[s] else np.zeros(0, int)
        q_pos.append(pos)
        cu.append(cu[-1] + pos.size)
    q_pos = np.concatenate(q_pos).astype(np.int32)
    cu = np.asarray(cu, np.int32)
    n_q = int(q_pos.size)
    q = _pool(rng, (max(1, n_q), n_q_heads, d), dtype)[:n_q]
    scale = scale_mult / math.sqrt(d)
    if late_outlier > 0:
        for s in range(n_streams):
            j = max(0, kv_lens[s] - 1 - min(40, kv_lens[s] // 3))
            slot = int(bt[s, j // 16]) * 16 + j % 16
            kc[slot] = (kc[slot].float() * late_outlier).to(kc.dtype)
    ref = oc.window_attn(hp.f64(q), hp.f64(kc), hp.f64(vc), cu, q_pos, bt, n_q_heads, scale)
    if poison:
        # cache rows past every stream's frontier hold NaN: they must never influence a result
        used = np.zeros(n_blocks * 16, bool)
        for s in range(n_streams):
            seg = q_pos[cu[s]: cu[s + 1]]
            if seg.size:
                j = np.arange(int(seg.max()) + 1)
                used[bt[s, j // 16] * 16 + j % 16] = True
        kc[torch.from_numpy(~used)] = float("nan")
        vc[torch.from_numpy(~used)] = float("nan")
    out = torch.full((max(1, n_q), n_q_heads, d), 7.0, dtype=q.dtype, device=DEV)
    kd, vd = kc.to(DEV), vc.to(DEV)
    code = cs.CS_BF16 if dtype == "bf16" else cs.CS_F32
    wsb = cs.cs_window_prefill_attn_workspace(n_q, n_streams, n_q_heads, n_kv_heads, d, max_blocks, code)
    ws = torch.randint(0, 255, (max(16, wsb),), dtype=torch.uint8, device=DEV)     # dirty workspace
    cs.cs_window_prefill_attn(q.to(DEV), kd, vd, torch.from_numpy(cu).to(DEV), torch.from_numpy(q_pos).to(DEV),
                              torch.tensor(kv_lens, dtype=torch.int32, device=DEV),
                              torch.from_numpy(bt).to(DEV), max_blocks, 16, out, n_q, n_streams, n_q_heads,
                              n_kv_heads, d, kd.stride(0), kd.stride(1), scale, code, ws, wsb)
    torch.cuda.synchronize()
    return hp.check_attention(out[:n_q].cpu(), ref, dtype)


PLAN_HDR_INTS = 32 + 32 * 8 * 64        # list offsets, row-tile count, end item; then one 32-int entry per (XCD, workgroup)


def _attention_plan(cs, cu, q_pos, kv_lens, bt, hq, hkv):
    """Runs the planning launch alone and returns (header ints, item descriptors [n, 8])."""
    n_streams, max_blocks, n_q = len(kv_lens), int(bt.shape[1]), int(q_pos.size)
    d = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a).astype(dt)).to(DEV)
    wsb = cs.cs_window_prefill_attn_workspace(n_q, n_streams, hq, hkv, 128, max_blocks, cs.CS_BF16)
    ws = torch.randint(0, 255, (wsb,), dtype=torch.uint8, device=DEV)
    cs.cs_window_prefill_attn(None, None, None, d(cu, np.int32), d(q_pos, np.int32), d(kv_lens, np.int32), d(bt, np.int32),
                              max_blocks, 16, None, n_q, n_streams, hq, hkv, 128, hkv * 128, 128, 0.1, cs.CS_BF16, ws, wsb,
                              cs.CS_ATTN_PLAN_ONLY)
    torch.cuda.synchronize()
    hdr = ws[: PLAN_HDR_INTS * 4].view(torch.int32).cpu().numpy()
    # behind the entries: the counters of the fused launch's barrier (18 words, 64 ints apart), then the items
    off = (((PLAN_HDR_INTS + 63) // 64 * 64 + 18 * 64) * 4 + 255) // 256 * 256
    n_items = int(hdr[8])
    items = ws[off: off + n_items * 32].view(torch.int32).cpu().numpy().reshape(n_items, 8)
    return hdr, items


@pytest.mark.parametrize("hq,hkv,kv_lens,n_qs", [
    (28, 4, [915], [425]),                                              # one stream, sweeps split over keys
    (32, 8, [300, 1, 640, 77], [100, 1, 333, 0]),                       # lists dealt by pair, short batches
    (8, 1, [513], [70]),
    (28, 4, [6033], [300]),
    (8, 2, [3000, 700, 40], [257, 64, 40]),
    (2, 1, [20] * 2100, [2] * 2100),
    (28, 4, [300 + 7 * i for i in range(40)], [60 + i for i in range(40)]),     # more items than workgroups
    (28, 4, [1100 + 13 * i for i in range(32)], [380 + 5 * i for i in range(32)]),
])
def test_attention_plan_is_a_valid_schedule(cs, hq, hkv, kv_lens, n_qs):
    """The planning launch alone (nothing computed, nothing that could fault on a bad schedule): the
    items cover every (stream, kv head, row tile) and its key tiles exactly once, every item lies on
    exactly one workgroup's chain inside its XCD's list, and each workgroup's header entry agrees
    with its chain.  Runs before the attention tests, which trust the plan."""
    say(f"attention plan: heads={hq}/{hkv} streams={len(kv_lens)} rows={sum(n_qs) * (hq // hkv)}")
    rng = np.random.default_rng(4000 + len(kv_lens) + sum(n_qs))
    g = hq // hkv
    nb = [-(-L // 16) for L in kv_lens]
    bt = np.zeros((len(kv_lens), max(nb) + 1), np.int32)
    ids, at = rng.permutation(sum(nb) + 3), 0
    for s in range(len(kv_lens)):
        bt[s, : nb[s]] = ids[at: at + nb[s]]
        at += nb[s]
    q_pos, cu = [], [0]
    for s in range(len(kv_lens)):
        q_pos.append(np.sort(rng.choice(kv_lens[s], size=n_qs[s], replace=False)) if n_qs[s] else np.zeros(0, int))
        cu.append(cu[-1] + n_qs[s])
    q_pos = np.concatenate(q_pos).astype(np.int64)
    hdr, items = _attention_plan(cs, np.asarray(cu), q_pos, np.asarray(kv_lens), bt, hq, hkv)
    lists = hdr[:9]
    assert lists[0] == 0 and np.all(np.diff(lists) >= 0) and lists[8] == items.shape[0]
    assert list(hdr[16:24]) == [0, 0, 0, 0, -1, 0, -1, -1]                 # the end item
    # ---- coverage: key ranges of a row tile's items tile [0, n_kt) exactly
    ranges = {}
    for it in items:
        q0, rows, r_tile, kvh_s, wg_max, kbe = (int(v) for v in it[:6])
        ranges.setdefault((kvh_s >> 8, kvh_s & 255, r_tile), []).append((kbe & 0xffff, kbe >> 16, q0, rows, wg_max))
    want = set()
    for s in range(len(kv_lens)):
        rows = n_qs[s] * g
        for t in range(-(-rows // 128)):
            last = min((t + 1) * 128, rows) - 1
            wg_max = int(q_pos[cu[s] + last // g])
            for kvh in range(hkv):
                want.add((s, kvh, t * 128))
                segs = sorted(ranges.get((s, kvh, t * 128), []))
                assert segs, (s, kvh, t)
                assert all(x[2] == cu[s] and x[3] == rows and x[4] == wg_max for x in segs)
                assert segs[0][0] == 0 and segs[-1][1] == wg_max // 64 + 1
                assert all(a[1] == b[0] and a[0] < a[1] for a, b in zip(segs, segs[1:])) and segs[-1][0] < segs[-1][1]
    assert set(ranges) == want
    assert hdr[9] == len(want)
    # ---- chains
    seen = np.zeros(items.shape[0], bool)
    for x in range(8):
        for j in range(64):
            e = hdr[32 + 32 * (64 * x + j): 32 + 32 * (64 * x + j) + 17]
            chain, i = [], int(e[0])
            while i >= 0:
                assert lists[x] <= i < lists[x + 1] and not seen[i], (x, j, i)
                seen[i] = True
                chain.append(i)
                i = int(items[i, 6])
            assert int(e[16]) == len(chain) and [int(v) for v in e[:3]] == (chain + [-1, -1, -1])[:3]
            if chain:
                first = items[chain[0]]
                assert np.array_equal(e[8:16], first)
                row, last_blk, kt0 = bt[int(first[3]) >> 8], int(first[4]) >> 4, int(first[5]) & 0xffff
                assert int(e[3]) == int(row[last_blk])
                assert [int(v) for v in e[4:8]] == [int(row[min(kt0 * 4 + i, last_blk)]) for i in range(4)]
            else:
                assert list(e[8:16]) == [0, 0, 0, 0, -1, 0, -1, -1]
    assert seen.all()


ATTN_CASES = [
    # dtype, Hq, Hkv, d, kv_lens, n_qs
    ("f32", 2, 1, 64, [452], [332]),
    ("f32", 4, 2, 128, [100, 37], [20, 37]),
    ("bf16", 28, 4, 128, [915], [425]),                       # 7 query heads per kv head
    ("bf16", 32, 8, 128, [300, 1, 640, 77], [100, 1, 333, 0]),  # a stream with no queries, one of length 1
    ("bf16", 4, 4, 64, [200, 129], [64, 129]),                # MHA, d = 64
    ("bf16", 8, 1, 128, [513], [70]),                         # 8-way group, ragged tail of one key
    ("bf16", 2, 1, 64, [1040], [18]),
    ("bf16", 28, 4, 128, [64, 65, 127, 128], [5, 9, 19, 37]),  # frontiers on tile edges
    ("bf16", 28, 4, 128, [6033], [300]),                      # long sweep, few rows: split over keys
    ("bf16", 8, 2, 128, [3000, 700, 40], [257, 64, 40]),      # split and unsplit row tiles in one launch
    ("bf16", 2, 1, 128, [20] * 2100, [2] * 2100),             # more streams than the planner sorts
    ("bf16", 28, 4, 128, [300 + 7 * i for i in range(40)], [60 + i for i in range(40)]),   # > 512 work items
]


# Rows whose maximum keeps moving: logits 4x / 8x wider than unit-scale data gives, or one key that
# dominates late in the sweep.  The online softmax then raises its reference maximum after an item's
# first tile (rescaling what it has accumulated), and the partial results of a split sweep meet with
# maxima far apart.  Also the group sizes between the configurations' 4 and 7 and the largest one.
ATTN_HARD_CASES = [
    # dtype, Hq, Hkv, d, kv_lens, n_qs, scale_mult, late_outlier
    ("bf16", 28, 4, 128, [915], [425], 4.0, 0.0),
    ("bf16", 28, 4, 128, [915], [425], 8.0, 0.0),
    ("bf16", 28, 4, 128, [6033], [300], 4.0, 0.0),               # split sweep, peaked rows
    ("bf16", 28, 4, 128, [6033], [300], 1.0, 6.0),               # split sweep, the last key range dominates
    ("bf16", 32, 8, 128, [700, 1300, 90], [300, 500, 60], 8.0, 0.0),
    ("bf16", 32, 8, 128, [700, 1300, 90], [300, 500, 60], 1.0, 5.0),
    ("bf16", 6, 2, 128, [800, 333], [200, 111], 1.0, 0.0),        # 3 query heads per kv head
    ("bf16", 16, 1, 128, [1000], [260], 1.0, 0.0),                # 16 query heads per kv head
    ("bf16", 16, 1, 128, [2500], [90], 4.0, 4.0),                 # ... split sweep, moving maximum
    ("bf16", 48, 16, 64, [400, 200], [100, 64], 4.0, 0.0),        # d = 64 path, 3 per group
    ("f32", 16, 1, 64, [300], [50], 8.0, 5.0),
]


@pytest.mark.parametrize("case", range(len(ATTN_HARD_CASES)))
def test_window_prefill_attn_moving_maximum_and_group_sizes(cs, case):
    dtype, hq, hkv, d, kv_lens, n_qs, mult, outlier = ATTN_HARD_CASES[case]
    say(f"window_prefill_attn hard case {case}: {dtype} heads={hq}/{hkv} d={d} kv={kv_lens} n_q={n_qs} "
        f"scale x{mult} outlier x{outlier}")
    stats = _attn_case(cs, np.random.default_rng(3500 + case), dtype, hq, hkv, d, kv_lens, n_qs,
                       scale_mult=mult, late_outlier=outlier)
    say(f"  -> {stats}")


@pytest.mark.parametrize("scale", [0.0, -0.1, float("inf"), float("nan")])
def test_window_prefill_attn_rejects_bad_scale(cs, scale):
    """A softmax scale that is not a positive finite number is an argument error (no launch)."""
    say(f"window_prefill_attn: softmax_scale = {scale} is rejected")
    z = torch.zeros((16, 4, 128), dtype=torch.bfloat16, device=DEV)
    kc = torch.zeros((64, 1, 128), dtype=torch.bfloat16, device=DEV)
    i32 = lambda v: torch.tensor(v, dtype=torch.int32, device=DEV)
    wsb = cs.cs_window_prefill_attn_workspace(16, 1, 4, 1, 128, 4, cs.CS_BF16)
    ws = torch.zeros((max(16, wsb),), dtype=torch.uint8, device=DEV)
    with pytest.raises(cs.CodecSightError) as exc:
        cs.cs_window_prefill_attn(z, kc, kc, i32([0, 16]), i32(list(range(16))), i32([64]), i32([[0, 1, 2, 3]]), 4, 16,
                                  torch.zeros_like(z), 16, 1, 4, 1, 128, 128, 128, scale, cs.CS_BF16, ws, wsb)
    assert exc.value.code == cs.CS_EINVAL


def test_window_prefill_attn_clamps_the_frontier_to_kv_len(cs):
    """A q_pos at or beyond its stream's kv_len is read as kv_len - 1: the call never indexes past
    the rows the block table defines (the cache past them holds NaN here)."""
    say("window_prefill_attn: q_pos beyond kv_len is clamped")
    rng = np.random.default_rng(77)
    hq, hkv, d, kv_len, n_q = 8, 2, 128, 200, 40
    nb = -(-kv_len // 16)
    bt = rng.permutation(nb + 5)[:nb].astype(np.int32)[None]
    kc, vc = _pool(rng, ((nb + 5) * 16, hkv, d), "bf16"), _pool(rng, ((nb + 5) * 16, hkv, d), "bf16")
    q = _pool(rng, (n_q, hq, d), "bf16")
    q_pos = np.sort(rng.choice(kv_len, n_q, replace=False)).astype(np.int32)
    bad = q_pos.copy()
    bad[-3:] = [kv_len, kv_len + 500, 2 ** 30]                     # non-decreasing, out of range
    good = q_pos.copy()
    good[-3:] = kv_len - 1
    cu = np.array([0, n_q], np.int32)
    scale = 1.0 / math.sqrt(d)
    ref = oc.window_attn(hp.f64(q), hp.f64(kc), hp.f64(vc), cu, good, bt, hq, scale)
    used = np.zeros((nb + 5) * 16, bool)
    j = np.arange(kv_len)
    used[bt[0, j // 16] * 16 + j % 16] = True
    kc[torch.from_numpy(~used)] = float("nan")
    vc[torch.from_numpy(~used)] = float("nan")
    for dtype, code in (("bf16", cs.CS_BF16),):
        out = torch.zeros((n_q, hq, d), dtype=torch.bfloat16, device=DEV)
        wsb = cs.cs_window_prefill_attn_workspace(n_q, 1, hq, hkv, d, nb, code)
        ws = torch.zeros((max(16, wsb),), dtype=torch.uint8, device=DEV)
        kd, vd = kc.to(DEV), vc.to(DEV)
        cs.cs_window_prefill_attn(q.to(DEV), kd, vd, torch.from_numpy(cu).to(DEV), torch.from_numpy(bad).to(DEV),
                                  torch.tensor([kv_len], dtype=torch.int32, device=DEV), torch.from_numpy(bt).to(DEV),
                                  nb, 16, out, n_q, 1, hq, hkv, d, kd.stride(0), kd.stride(1), scale, code, ws, wsb)
        torch.cuda.synchronize()
        say(f"  -> {hp.check_attention(out.cpu(), ref, dtype)}")


@pytest.mark.parametrize("case", range(len(ATTN_CASES)))
def test_window_prefill_attn(cs, case):
    dtype, hq, hkv, d, kv_lens, n_qs = ATTN_CASES[case]
    say(f"window_prefill_attn case {case}: {dtype} heads={hq}/{hkv} d={d} kv={kv_lens} n_q={n_qs}")
    stats = _attn_case(cs, np.random.default_rng(3000 + case), dtype, hq, hkv, d, kv_lens, n_qs)
    say(f"  -> {stats}")


def test_attention_plan_modes(cs):
    """The work plan depends on cu_q / q_pos only: built by one call (or by a plan-only call), it
    serves later calls on other Q / K / V (the decoder layers of a step) in REUSE mode."""
    say("window_prefill_attn: plan built once, reused for other layers; plan-only call")
    rng = np.random.default_rng(41)
    hq, hkv, d = 28, 4, 128
    kv_lens = [700, 90, 1300, 260, 33]
    n_qs = [120, 90, 300, 7, 20]
    n_streams = len(kv_lens)
    nb = [(-(-L // 16)) for L in kv_lens]
    max_blocks = max(nb)
    ids = rng.permutation(sum(nb))
    bt = np.zeros((n_streams, max_blocks), np.int32)
    at = 0
    for s in range(n_streams):
        bt[s, : nb[s]] = ids[at: at + nb[s]]
        at += nb[s]
    q_pos = np.concatenate([np.sort(rng.choice(kv_lens[s], n_qs[s], replace=False)) for s in range(n_streams)]).astype(np.int32)
    cu = np.concatenate([[0], np.cumsum(n_qs)]).astype(np.int32)
    n_q = int(q_pos.size)
    scale = 1.0 / math.sqrt(d)
    layers = []
    for _ in range(3):
        q = _pool(rng, (n_q, hq, d), "bf16")
        kc = _pool(rng, (sum(nb) * 16, hkv, d), "bf16")
        vc = _pool(rng, (sum(nb) * 16, hkv, d), "bf16")
        layers.append((q, kc, vc, oc.window_attn(hp.f64(q), hp.f64(kc), hp.f64(vc), cu, q_pos, bt, hq, scale)))
    wsb = cs.cs_window_prefill_attn_workspace(n_q, n_streams, hq, hkv, d, max_blocks, cs.CS_BF16)
    meta = (torch.from_numpy(cu).to(DEV), torch.from_numpy(q_pos).to(DEV),
            torch.tensor(kv_lens, dtype=torch.int32, device=DEV), torch.from_numpy(bt).to(DEV))

    def run(layer, ws, mode):
        q, kc, vc, ref = layers[layer]
        out = torch.full((n_q, hq, d), 7.0, dtype=torch.bfloat16, device=DEV)
        kd, vd = kc.to(DEV), vc.to(DEV)
        cs.cs_window_prefill_attn(q.to(DEV), kd, vd, *meta, max_blocks, 16, out, n_q, n_streams, hq, hkv, d,
                                  kd.stride(0), kd.stride(1), scale, cs.CS_BF16, ws, wsb, mode)
        torch.cuda.synchronize()
        return hp.check_attention(out.cpu(), ref, "bf16")

    ws = torch.randint(0, 255, (wsb,), dtype=torch.uint8, device=DEV)
    run(0, ws, cs.CS_ATTN_PLAN_BUILD)
    run(1, ws, cs.CS_ATTN_PLAN_REUSE)
    run(2, ws, cs.CS_ATTN_PLAN_REUSE)
    run(0, ws, cs.CS_ATTN_PLAN_REUSE)
    ws2 = torch.randint(0, 255, (wsb,), dtype=torch.uint8, device=DEV)
    cs.cs_window_prefill_attn(None, None, None, *meta, max_blocks, 16, None, n_q, n_streams, hq, hkv, d,
                              hkv * d, d, scale, cs.CS_BF16, ws2, wsb, cs.CS_ATTN_PLAN_ONLY)
    run(2, ws2, cs.CS_ATTN_PLAN_REUSE)


FUSED_CASES = [
    # dtype, Hq, Hkv, d, kv_lens, n_qs
    ("bf16", 28, 4, 128, [915], [425]),                        # split sweeps (merge kernel after the fused launch)
    ("bf16", 32, 8, 128, [300, 1, 640, 77], [100, 1, 333, 0]),
    ("bf16", 28, 4, 128, [1100 + 13 * i for i in range(32)], [380 + 5 * i for i in range(32)]),   # all 512 workgroups busy
    ("bf16", 8, 2, 128, [3000, 700, 40], [257, 64, 40]),
    ("bf16", 4, 4, 64, [200, 129], [64, 129]),                 # head_dim 64: two launches behind the one call
    ("f32", 2, 1, 64, [452], [332]),                           # fp32: two launches behind the one call
]


@pytest.mark.parametrize("case", range(len(FUSED_CASES)))
def test_refresh_prefill_attn_equals_scatter_then_attention(cs, case):
    """The fused call against the oracle's refresh write followed by its attention (the executed
    tokens' own K/V rows go to the slots of their window positions first, so every query sees fresh
    rows written by other workgroups of the same launch), and bit for bit against the two separate
    calls; repeated on the same workspace with the plan reused and other data."""
    dtype, hq, hkv, d, kv_lens, n_qs = FUSED_CASES[case]
    say(f"refresh_prefill_attn case {case}: {dtype} heads={hq}/{hkv} d={d} kv={kv_lens} n_q={n_qs}")
    rng = np.random.default_rng(6100 + case)
    n_streams = len(kv_lens)
    nb = [(-(-L // 16)) for L in kv_lens]
    max_blocks = max(nb) + 1
    n_blocks = sum(nb) + 3
    ids = rng.permutation(n_blocks)
    bt = np.zeros((n_streams, max_blocks), np.int32)
    at = 0
    for s in range(n_streams):
        bt[s, : nb[s]] = ids[at: at + nb[s]]
        at += nb[s]
    q_pos, cu = [], [0]
    for s in range(n_streams):
        pos = np.sort(rng.choice(kv_lens[s], size=n_qs[s], replace=False)) if n_qs[s] else np.zeros(0, int)
        q_pos.append(pos)
        cu.append(cu[-1] + pos.size)
    q_pos = np.concatenate(q_pos).astype(np.int32)
    cu = np.asarray(cu, np.int32)
    n_q = int(q_pos.size)
    slot = np.concatenate([bt[s, q_pos[cu[s]: cu[s + 1]] // 16].astype(np.int64) * 16 + q_pos[cu[s]: cu[s + 1]] % 16
                           for s in range(n_streams)]).astype(np.int32)
    pad = 37                                                     # list padded beyond the executed rows
    slot_p = np.concatenate([slot, np.full(pad, -1, np.int32)])
    scale = 1.0 / math.sqrt(d)
    code = cs.CS_BF16 if dtype == "bf16" else cs.CS_F32
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    wsb = cs.cs_window_prefill_attn_workspace(n_q + pad, n_streams, hq, hkv, d, max_blocks, code)
    ws = torch.randint(0, 255, (max(64, wsb),), dtype=torch.uint8, device=DEV)
    dev = lambda a: torch.from_numpy(a).to(DEV)
    meta = (dev(cu), dev(np.concatenate([q_pos, np.zeros(pad, np.int32)])), torch.tensor(kv_lens, dtype=torch.int32, device=DEV),
            dev(bt))
    for rep, mode in enumerate((cs.CS_ATTN_PLAN_BUILD, cs.CS_ATTN_PLAN_REUSE)):
        kc, vc = _pool(rng, (n_blocks * 16, hkv, d), dtype), _pool(rng, (n_blocks * 16, hkv, d), dtype)
        kn, vn = _pool(rng, (n_q + pad, hkv, d), dtype), _pool(rng, (n_q + pad, hkv, d), dtype)
        q = _pool(rng, (n_q + pad, hq, d), dtype)
        # oracle: refresh write, then attention over the cache it leaves
        raw = torch.int16 if dtype == "bf16" else torch.int32
        k_ref, v_ref = kc.clone(), vc.clone()
        oc.scatter(k_ref.view(raw).numpy(), kn.view(raw).numpy(), slot_p)
        oc.scatter(v_ref.view(raw).numpy(), vn.view(raw).numpy(), slot_p)
        ref = oc.window_attn(hp.f64(q[:n_q]), hp.f64(k_ref), hp.f64(v_ref), cu, q_pos, bt, hq, scale)
        # the two separate calls
        k2, v2 = kc.to(DEV), vc.to(DEV)
        out2 = torch.full((n_q + pad, hq, d), 7.0, dtype=tdt, device=DEV)
        ws2 = torch.zeros_like(ws)
        cs.cs_kv_refresh_scatter(kn.to(DEV), vn.to(DEV), dev(slot_p), k2, v2, n_q + pad, hkv, d, k2.stride(0), k2.stride(1), code)
        cs.cs_window_prefill_attn(q.to(DEV), k2, v2, *meta, max_blocks, 16, out2, n_q + pad, n_streams, hq, hkv, d,
                                  k2.stride(0), k2.stride(1), scale, code, ws2, wsb)
        # the fused call
        k1, v1 = kc.to(DEV), vc.to(DEV)
        out1 = torch.full((n_q + pad, hq, d), 7.0, dtype=tdt, device=DEV)
        cs.cs_refresh_prefill_attn(kn.to(DEV), vn.to(DEV), dev(slot_p), n_q + pad, q.to(DEV), k1, v1, *meta, max_blocks, 16,
                                   out1, n_q + pad, n_streams, hq, hkv, d, k1.stride(0), k1.stride(1), scale, code,
                                   ws, wsb, mode)
        torch.cuda.synchronize()
        if dtype == "bf16" and d == 128:
            assert cs.cs_attn_status(ws) == 0, "the launch-wide barrier ran into its bound"
        assert torch.equal(k1.cpu().view(raw), k_ref.view(raw)) and torch.equal(v1.cpu().view(raw), v_ref.view(raw))
        assert torch.equal(out1.view(raw), out2.view(raw)), f"fused and separate calls differ (pass {rep})"
        assert torch.all(out1[n_q:].float() == 7.0)
        say(f"  pass {rep}: {hp.check_attention(out1[:n_q].cpu(), ref, dtype)}")


def test_fused_step_equals_the_step_of_separate_calls(cs):
    """The whole device-planned step with the refresh write inside the attention launch: cache and
    outputs bit-equal to the step that queues the two calls, also when replayed from a HIP graph."""
    w = synth.small_variant(synth.CFG2, n_streams=3, n_layers=3)
    say(f"fused step: {w.name} streams={w.n_streams} layers={w.n_layers}")
    data = engine.assemble_step(w, engine.hip_scorer, device="cpu")
    n_reuse, n_q = data.info["n_reuse"], data.info["n_q"]
    plain = engine.DeviceStep(data, reuse_cap=n_reuse + 64, q_cap=n_q + 64)
    fused = engine.DeviceStep(data, reuse_cap=n_reuse + 64, q_cap=n_q + 64, fused=True)
    plain.run()
    fused.run()
    assert fused.attention_status() == 0
    for name in ("k_pool", "v_pool", "out"):
        assert torch.equal(getattr(plain, name).view(torch.int16), getattr(fused, name).view(torch.int16)), name
    k0, v0 = data.k_pool.to(DEV), data.v_pool.to(DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fused.run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fused.run()
    for rep in range(3):
        fused.k_pool.copy_(k0); fused.v_pool.copy_(v0); fused.out.zero_()
        scratch = torch.randn(1 << 20, device=DEV).sum().item()
        assert math.isfinite(scratch)
        graph.replay()
        assert fused.attention_status() == 0
        for name in ("k_pool", "v_pool", "out"):
            assert torch.equal(getattr(plain, name).view(torch.int16), getattr(fused, name).view(torch.int16)), (rep, name)


@pytest.mark.parametrize("layers_per_call", [1, 2, 5])
def test_step_with_rerotation_beside_the_layer_loop_equals_the_serial_step(cs, layers_per_call):
    """The position correction queued on a second stream, a few layers per call, each layer's
    attention waiting for the call that covers it: cache and outputs bit-equal to the step that
    corrects all layers first, eagerly and replayed from a HIP graph (the fork and join are edges
    of the captured graph)."""
    w = synth.small_variant(synth.CFG2, n_streams=3, n_layers=5)
    say(f"overlapped step: {w.name} streams={w.n_streams} layers={w.n_layers} layers per call={layers_per_call}")
    data = engine.assemble_step(w, engine.hip_scorer, device="cpu")
    n_reuse, n_q = data.info["n_reuse"], data.info["n_q"]
    serial = engine.DeviceStep(data, reuse_cap=n_reuse + 64, q_cap=n_q + 64, overlap=False)
    beside = engine.DeviceStep(data, reuse_cap=n_reuse + 64, q_cap=n_q + 64, overlap=True, layers_per_rerotate=layers_per_call)
    assert not serial.overlap and beside.overlap
    serial.run()
    beside.run()
    torch.cuda.synchronize()
    for name in ("k_pool", "v_pool", "out"):
        assert torch.equal(getattr(serial, name).view(torch.int16), getattr(beside, name).view(torch.int16)), name
    k0, v0 = data.k_pool.to(DEV), data.v_pool.to(DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        beside.run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        beside.run()
    for rep in range(3):
        beside.k_pool.copy_(k0); beside.v_pool.copy_(v0); beside.out.zero_()
        assert math.isfinite(torch.randn(1 << 20, device=DEV).sum().item())
        graph.replay()
        torch.cuda.synchronize()
        for name in ("k_pool", "v_pool", "out"):
            assert torch.equal(getattr(serial, name).view(torch.int16), getattr(beside, name).view(torch.int16)), (rep, name)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_attention_nothing_pruned_equals_full_causal(cs, dtype):
    """With every token a query the call is plain causal attention (1040-token tiny window)."""
    say(f"window_prefill_attn: all 1040 tokens are queries, {dtype}")
    stats = _attn_case(cs, np.random.default_rng(11), dtype, 2, 1, 64, [1040], [1040], all_queries=True)
    say(f"  -> {stats}")


def test_attention_properties_on_gpu(cs):
    """Constant values come back unchanged; a query at index 0 returns V_0."""
    say("window_prefill_attn: V == 1 and q_pos == 0 properties (bf16)")
    rng = np.random.default_rng(5)
    n_q, hq, hkv, d = 50, 8, 2, 128
    kc = _pool(rng, (512, hkv, d), "bf16").to(DEV)
    vc = torch.ones((512, hkv, d), dtype=torch.bfloat16, device=DEV)
    q = _pool(rng, (n_q, hq, d), "bf16").to(DEV)
    q_pos = torch.from_numpy(np.sort(rng.choice(500, n_q, replace=False)).astype(np.int32)).to(DEV)
    q_pos[0] = 0
    bt = torch.arange(32, dtype=torch.int32, device=DEV).reshape(1, 32)
    out = torch.zeros_like(q)
    args = (torch.tensor([0, n_q], dtype=torch.int32, device=DEV), q_pos,
            torch.tensor([500], dtype=torch.int32, device=DEV), bt, 32, 16)
    wsb = cs.cs_window_prefill_attn_workspace(n_q, 1, hq, hkv, d, 32, cs.CS_BF16)
    ws = torch.zeros((max(16, wsb),), dtype=torch.uint8, device=DEV)
    cs.cs_window_prefill_attn(q, kc, vc, *args, out, n_q, 1, hq, hkv, d, hkv * d, d, 0.09, cs.CS_BF16, ws, wsb)
    torch.cuda.synchronize()
    assert torch.all(out.float() == 1.0)
    vr = _pool(rng, (512, hkv, d), "bf16").to(DEV)
    cs.cs_window_prefill_attn(q, kc, vr, *args, out, n_q, 1, hq, hkv, d, hkv * d, d, 0.09, cs.CS_BF16, ws, wsb)
    torch.cuda.synchronize()
    for h in range(hq):
        assert torch.equal(out[0, h], vr[0, h // (hq // hkv)])


# =============================================================================== (p) refresh plan
def _plan_inputs(rng, n_streams, window, stride, t_per, n_text, p_iframe, p_empty, shuffle=True):
    """Random cached windows + new frames: counts in 0..T (some frames empty), I-frames anywhere."""
    def counts(n):
        c = rng.integers(0, t_per + 1, size=(n_streams, n)).astype(np.int32)
        c[rng.random((n_streams, n)) < p_empty] = 0
        return c
    old_types = (rng.random((n_streams, window)) < p_iframe).astype(np.uint8)
    new_types = (rng.random((n_streams, stride)) < p_iframe).astype(np.uint8)
    old_counts, new_counts = counts(window), counts(stride)
    old_len = old_counts.sum(1) + n_text
    new_len = old_counts[:, stride:].sum(1) + new_counts.sum(1) + n_text
    nb_old, nb_new = (old_len + 15) // 16, (new_len + 15) // 16
    mb_old, mb_new = max(1, int(nb_old.max(initial=0))), max(1, int(nb_new.max(initial=0)))
    total = int(nb_old.sum() + nb_new.sum())
    ids = rng.permutation(total + 5) if shuffle else np.arange(total + 5)
    bt_old = np.full((n_streams, mb_old), -3, np.int32)
    bt_new = np.full((n_streams, mb_new), -3, np.int32)
    at = 0
    for s in range(n_streams):
        bt_old[s, : nb_old[s]] = ids[at: at + nb_old[s]]; at += int(nb_old[s])
        bt_new[s, : nb_new[s]] = ids[at: at + nb_new[s]]; at += int(nb_new[s])
    return old_types, old_counts, new_types, new_counts, bt_old, bt_new


def _plan_oracle(old_types, old_counts, new_types, new_counts, bt_old, bt_new, n_text, t_per):
    from oracle import plan_oracle as po
    keys = ("src_slot", "dst_slot", "delta", "q_pos", "q_slot", "q_kind")
    cat = {k: [] for k in keys}
    cu_q, kv_len = [0], []
    for s in range(old_types.shape[0]):
        pl = po.plan_stream(old_types[s].tolist(), old_counts[s].tolist(), new_types[s].tolist(),
                            new_counts[s].tolist(), n_text, t_per, bt_old[s], bt_new[s])
        for k in keys:
            cat[k] += pl[k]
        cu_q.append(cu_q[-1] + len(pl["q_pos"]))
        kv_len.append(pl["kv_len"])
    out = {k: np.asarray(v, np.int64) for k, v in cat.items()}
    out["cu_q"], out["kv_len"] = np.asarray(cu_q, np.int64), np.asarray(kv_len, np.int64)
    return out


def _plan_gpu(cs, old_types, old_counts, new_types, new_counts, bt_old, bt_new, n_text, t_per, reuse_cap, q_cap):
    n_streams, window = old_types.shape
    stride = new_types.shape[1]
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    kept_off = np.concatenate([[0], np.cumsum(new_counts.reshape(-1))]).astype(np.int32) + 11   # any base
    fill = lambda n, v, dt=torch.int32: torch.full((max(1, n),), v, dtype=dt, device=DEV)
    o = dict(src_slot=fill(reuse_cap + 3, -77), dst_slot=fill(reuse_cap + 3, -77), delta=fill(reuse_cap + 3, -77),
             q_pos=fill(q_cap + 3, -77), q_slot=fill(q_cap + 3, -77), q_kind=fill(q_cap + 3, 99, torch.uint8),
             cu_q=fill(n_streams + 1, -77), kv_len=fill(n_streams, -77),
             out_types=fill(n_streams * window, 99, torch.uint8), out_counts=fill(n_streams * window, -77),
             totals=fill(4, -77))
    nbytes = cs.cs_plan_refresh_workspace(n_streams, window)
    ws = torch.randint(0, 255, (max(16, nbytes),), dtype=torch.uint8, device=DEV)           # dirty workspace
    cs.cs_plan_refresh(d(old_types), d(old_counts), d(new_types), d(kept_off), d(bt_old), bt_old.shape[1],
                       d(bt_new), bt_new.shape[1], n_streams, window, stride, n_text, t_per, reuse_cap, q_cap,
                       o["src_slot"], o["dst_slot"], o["delta"], o["q_pos"], o["q_slot"], o["q_kind"], o["cu_q"],
                       o["kv_len"], o["out_types"], o["out_counts"], o["totals"], ws if nbytes else None, nbytes)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in o.items()}


def _check_plan(got, want, old_types, old_counts, new_types, new_counts, reuse_cap, q_cap, flags=0):
    n_streams, window = old_types.shape
    stride = new_types.shape[1]
    n_reuse, n_q = int(want["src_slot"].size), int(want["q_pos"].size)
    assert got["totals"].tolist() == [n_reuse, n_q, flags, 0]
    assert np.array_equal(got["cu_q"], np.minimum(want["cu_q"], q_cap))     # clamped when the capacity is short
    assert np.array_equal(got["kv_len"][:n_streams], want["kv_len"])
    r, q = min(n_reuse, reuse_cap), min(n_q, q_cap)
    for k in ("src_slot", "dst_slot", "delta"):
        assert np.array_equal(got[k][:r], want[k][:r]), k
        assert np.all(got[k][r:reuse_cap] == (0 if k == "delta" else -1)), k          # padding
        assert np.all(got[k][reuse_cap:] == -77), k                                    # past the capacity: untouched
    for k in ("q_pos", "q_slot", "q_kind"):
        assert np.array_equal(got[k][:q], want[k][:q]), k
        assert np.all(got[k][q:q_cap] == {"q_pos": 0, "q_slot": -1, "q_kind": 255}[k]), k
        assert np.all(got[k][q_cap:] == (99 if k == "q_kind" else -77)), k
    if n_streams:
        types = np.concatenate([old_types[:, stride:], new_types], axis=1)
        counts = np.concatenate([old_counts[:, stride:], new_counts], axis=1)
        assert np.array_equal(got["out_types"].reshape(n_streams, window), types)
        assert np.array_equal(got["out_counts"].reshape(n_streams, window), counts)


PLAN_CASES = [
    # streams, window, stride, T, n_text, p_iframe, p_empty, slack
    (1, 4, 1, 16, 4, 0.3, 0.0, 0),
    (3, 8, 1, 256, 64, 0.15, 0.1, 0),
    (5, 8, 2, 64, 0, 0.2, 0.3, 7),
    (2, 16, 16, 40, 9, 0.2, 0.0, 300),           # stride = window: nothing overlaps, nothing reused
    (4, 70, 3, 19, 5, 0.1, 0.2, 1),              # more than 64 frames: the per-stream scan carries across chunks
    (2, 200, 130, 7, 1, 0.5, 0.1, 0),            # more than 64 departing frames
    (1100, 3, 1, 5, 2, 0.3, 0.3, 513),           # more than 1024 streams: the stream scan carries across chunks
    (64, 8, 1, 256, 32, 0.125, 0.0, 256),
    (7, 6, 2, 33, 3, 1.0, 0.0, 0),               # every overlap frame an anchor: no reused row
    (7, 6, 2, 33, 3, 0.0, 0.0, 0),               # no anchor
    (3, 5, 2, 12, 0, 0.3, 1.0, 4),               # every frame empty, no text: no rows at all
]


@pytest.mark.parametrize("case", range(len(PLAN_CASES)))
def test_plan_refresh(cs, case):
    """Every list of the device plan equals the oracle's, bit for bit; padding and totals as declared."""
    n_streams, window, stride, t_per, n_text, p_i, p_e, slack = PLAN_CASES[case]
    say(f"plan_refresh case {case}: streams={n_streams} W={window} S={stride} T={t_per} text={n_text}")
    rng = np.random.default_rng(7000 + case)
    ins = _plan_inputs(rng, n_streams, window, stride, t_per, n_text, p_i, p_e)
    want = _plan_oracle(*ins, n_text, t_per)
    reuse_cap, q_cap = int(want["src_slot"].size) + slack, int(want["q_pos"].size) + slack
    got = _plan_gpu(cs, *ins, n_text, t_per, reuse_cap, q_cap)
    _check_plan(got, want, *ins[:4], reuse_cap, q_cap)
    say(f"  reused rows {want['src_slot'].size}, executed rows {want['q_pos'].size}")


def test_plan_refresh_no_streams(cs):
    say("plan_refresh with an empty batch")
    z8, z32 = np.zeros((0, 4), np.uint8), np.zeros((0, 4), np.int32)
    got = _plan_gpu(cs, z8, z32, np.zeros((0, 1), np.uint8), np.zeros((0, 1), np.int32), np.zeros((0, 1), np.int32),
                    np.zeros((0, 1), np.int32), 4, 16, 5, 6)
    assert got["totals"].tolist() == [0, 0, 0, 0] and got["cu_q"][0] == 0
    assert np.all(got["src_slot"][:5] == -1) and np.all(got["q_slot"][:6] == -1)


def test_plan_refresh_reports_what_does_not_fit(cs):
    """Capacities or block-table rows that are too short raise flags; nothing is written outside
    the capacities and no slot is formed from a missing block-table entry."""
    say("plan_refresh: capacities and block tables too small")
    rng = np.random.default_rng(7100)
    n_text, t_per = 8, 32
    ins = _plan_inputs(rng, 6, 8, 1, t_per, n_text, 0.15, 0.0)
    want = _plan_oracle(*ins, n_text, t_per)
    n_reuse, n_q = int(want["src_slot"].size), int(want["q_pos"].size)
    got = _plan_gpu(cs, *ins, n_text, t_per, n_reuse - 10, n_q)
    _check_plan(got, want, *ins[:4], n_reuse - 10, n_q, flags=1)
    got = _plan_gpu(cs, *ins, n_text, t_per, n_reuse, n_q // 2)
    _check_plan(got, want, *ins[:4], n_reuse, n_q // 2, flags=2)
    got = _plan_gpu(cs, *ins, n_text, t_per, 0, 0)
    _check_plan(got, want, *ins[:4], 0, 0, flags=3)
    # the new block-table rows cut to two blocks: indices from 32 on have no slot
    old_types, old_counts, new_types, new_counts, bt_old, bt_new = ins
    got = _plan_gpu(cs, old_types, old_counts, new_types, new_counts, bt_old, bt_new[:, :2].copy(), n_text, t_per,
                    n_reuse, n_q)
    assert got["totals"].tolist() == [n_reuse, n_q, 4, 0]
    lost_q = want["q_pos"] >= 32
    assert np.array_equal(got["q_pos"][:n_q], np.minimum(want["q_pos"], 31))       # pulled back onto the row
    assert np.all(got["q_slot"][:n_q][lost_q] == -1)
    assert np.array_equal(got["q_slot"][:n_q][~lost_q], want["q_slot"][~lost_q])
    lost_r = got["dst_slot"][:n_reuse] < 0
    assert lost_r.any() and np.all(got["src_slot"][:n_reuse][lost_r] == -1)
    assert np.array_equal(got["src_slot"][:n_reuse][~lost_r], want["src_slot"][~lost_r])
    assert np.array_equal(got["dst_slot"][:n_reuse][~lost_r], want["dst_slot"][~lost_r])


def test_plan_refresh_matches_the_host_planner_on_a_workload(cs):
    """The product's own host planner and the device planner agree on a workload-shaped batch."""
    w = synth.small_variant(synth.CFG4, n_streams=16)
    say(f"plan_refresh vs host planner: {w.name}")
    data = engine.assemble_step(w, engine.hip_scorer, device="cpu", with_tensors=False)
    p, old = data.plan, data.old_layout
    new_counts = p.layout.counts[:, w.window - w.stride:]
    new_types = p.layout.frame_type[:, w.window - w.stride:]
    got = _plan_gpu(cs, old.frame_type, old.counts, new_types, new_counts, old.block_table, p.layout.block_table,
                    w.n_text, w.tokens_per_frame, p.src_slot.size + 100, p.q_pos.size + 100)
    for k in ("src_slot", "dst_slot", "delta"):
        assert np.array_equal(got[k][: p.src_slot.size], getattr(p, k)), k
    for k in ("q_pos", "q_slot", "q_kind"):
        assert np.array_equal(got[k][: p.q_pos.size], getattr(p, k)), k
    assert np.array_equal(got["cu_q"], p.cu_q) and np.array_equal(got["kv_len"], p.kv_len)


# =============================================================================== whole step
def _oracle_step(data_o: engine.StepData, p: hp.OraclePlan, layers):
    """b -> c -> d with oracle pieces on host copies of the inputs, on the plan oracle's row lists;
    returns per-layer results."""
    w = data_o.workload
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    k_pool, v_pool = data_o.k_pool.clone(), data_o.v_pool.clone()
    k_rows, v_rows = oc.rerotate(hp.f64(k_pool[layers]), hp.f64(v_pool[layers]), p.src_slot, p.dst_slot,
                                 p.delta, w.rope_base)
    dst = torch.from_numpy(p.dst_slot.astype(np.int64))
    outs = {}
    for i, layer in enumerate(layers):
        k_pool[layer][dst] = hp.round_like(k_rows[:, i], tdt)
        v_pool[layer][dst] = hp.round_like(v_rows[:, i], tdt)
        raw = torch.int16 if w.dtype == "bf16" else torch.int32
        oc.scatter(k_pool[layer].view(raw).numpy(), data_o.k_new[layer].view(raw).numpy(), p.q_slot)
        oc.scatter(v_pool[layer].view(raw).numpy(), data_o.v_new[layer].view(raw).numpy(), p.q_slot)
        outs[layer] = oc.window_attn(hp.f64(data_o.q[layer]), hp.f64(k_pool[layer]), hp.f64(v_pool[layer]),
                                     p.cu_q, p.q_pos, p.block_table, w.n_q_heads, data_o.softmax_scale)
    return k_rows, k_pool, v_pool, outs


STEP_WORKLOADS = [
    synth.CFG0,
    synth.small_variant(synth.CFG1, n_layers=2),
    synth.small_variant(synth.CFG2, n_streams=3, n_layers=2),
    synth.small_variant(synth.CFG4, n_streams=4, n_layers=2),
]


@pytest.mark.parametrize("wi", range(len(STEP_WORKLOADS)))
def test_whole_step_against_oracle(cs, wi):
    """score -> plan -> re-rotate -> refresh write -> attention on a workload-shaped step; the HIP
    path and the oracle each run the whole chain from the same seeded inputs."""
    w = STEP_WORKLOADS[wi]
    say(f"whole step: {w.name} streams={w.n_streams} layers={w.n_layers}")
    data_g = engine.assemble_step(w, engine.hip_scorer, device="cpu")
    data_o = engine.assemble_step(w, hp.oracle_scorer, device="cpu")
    # (a) the two assemblies agree bit for bit (history scoring on the GPU vs the oracle)
    assert np.array_equal(data_g.old_layout.counts, data_o.old_layout.counts)
    assert np.array_equal(data_g.new_layout.counts, data_o.new_layout.counts)
    assert np.array_equal(data_g.new_layout.block_table, data_o.new_layout.block_table)
    assert np.array_equal(data_g.acc_in, data_o.acc_in)
    say(f"  sizes: {data_g.info}")
    plan = hp.OraclePlan(data_o)
    step = engine.DeviceStep(data_g)
    step.run()
    torch.cuda.synchronize()
    assert step.scoring_status() == 0
    hp.assert_device_plan(step, plan)                         # (p) the refresh plan, entry for entry
    # (a) on the step's own frames
    keep_w, idx_w, off_w, acc_w = hp.oracle_scorer(data_o.mv, data_o.sad, data_o.frame_type, data_o.cu_frames,
                                                   data_o.acc_in, w, w.tau_mv_sq, w.tau_sad)
    assert np.array_equal(step.keep.cpu().numpy(), keep_w)
    assert np.array_equal(step.kept_off.cpu().numpy(), off_w)
    assert np.array_equal(step.kept_idx.cpu().numpy()[: idx_w.size], idx_w)
    assert np.array_equal(step.acc.cpu().numpy() != 0, acc_w != 0)
    layers = list(range(w.n_layers))
    k_rows, k_pool_o, v_pool_o, outs = _oracle_step(data_o, plan, layers)
    dst = torch.from_numpy(plan.dst_slot.astype(np.int64))
    got_rows = step.k_pool.cpu()[:, dst].permute(1, 0, 2, 3).contiguous()
    say(f"  rerotate: {hp.check_rerotated(got_rows, k_rows, w.dtype)}")
    # (c) executed rows are bit-equal to the new K/V; values of reused rows are bit-equal copies
    qs = torch.from_numpy(plan.q_slot.astype(np.int64))
    assert torch.equal(step.k_pool.cpu()[:, qs], data_o.k_new) and torch.equal(step.v_pool.cpu()[:, qs], data_o.v_new)
    assert torch.equal(step.v_pool.cpu(), v_pool_o)
    for layer in layers:
        say(f"  attention layer {layer}: {hp.check_attention(step.out[layer].cpu(), outs[layer], w.dtype)}")


@pytest.mark.parametrize("wi,slack", [(0, 0), (1, 0), (1, 300), (2, 1000), (3, 77)])
def test_device_planned_step_equals_host_planned_step(cs, wi, slack):
    """score -> plan on the device -> re-rotate -> refresh write -> attention with nothing passing
    through the host, lists padded to capacities: the cache ends bit-equal to the host-planned
    step's (itself checked against the oracle above) and attention agrees (bit-equal when the
    capacities equal the row counts, since then the launches are identical)."""
    w = STEP_WORKLOADS[wi]
    say(f"device-planned step: {w.name} streams={w.n_streams} layers={w.n_layers} slack={slack}")
    data = engine.assemble_step(w, engine.hip_scorer, device="cpu")
    host = engine.DeviceStep(data, host_plan=True)
    host.run()
    n_reuse, n_q = data.info["n_reuse"], data.info["n_q"]
    devp = engine.DevicePlannedStep(data, reuse_cap=n_reuse + slack, q_cap=n_q + slack)
    devp.run()
    torch.cuda.synchronize()
    assert devp.totals.cpu().tolist() == [n_reuse, n_q, 0, 0]
    for name in ("src_slot", "dst_slot", "delta"):
        assert torch.equal(getattr(devp, name)[:n_reuse], getattr(host, name)), name
    for name in ("q_pos", "q_slot"):
        assert torch.equal(getattr(devp, name)[:n_q], getattr(host, name)), name
    assert torch.equal(devp.cu_q, host.cu_q) and torch.equal(devp.kv_len, host.kv_len)
    assert torch.equal(devp.k_pool.view(torch.uint8), host.k_pool.view(torch.uint8))
    assert torch.equal(devp.v_pool.view(torch.uint8), host.v_pool.view(torch.uint8))
    a, b = devp.out[:, :n_q].float().cpu(), host.out.float().cpu()
    if slack == 0:
        assert torch.equal(a, b)
    else:
        assert float((a - b).abs().max()) <= (2e-2 if w.dtype == "bf16" else 1e-4)
    assert not devp.out[:, n_q:].any()                           # rows past the executed rows are not written


def test_frontend_to_attention_chain_against_oracle_chain(cs):
    """Decoder output in, attention output out, nothing through the host in between: block
    projection, residual proxy, scoring with rescue, refresh plan, position correction, and per
    layer refresh write + attention, queued back to back on capacity-sized lists.  The oracle runs
    the same chain stage by stage from the same inputs."""
    from oracle import plan_oracle as plo
    from oracle import projection_oracle as pjo
    from oracle import residual_oracle as rso
    w = synth.small_variant(synth.CFG2, n_streams=2, n_layers=2)
    say(f"front end -> attention chain: {w.name} streams={w.n_streams} layers={w.n_layers}")
    data = engine.assemble_frontend_step(w, engine.hip_scorer, device="cpu")
    data_o = engine.assemble_frontend_step(w, hp.oracle_scorer, device="cpu")
    assert np.array_equal(data.old_layout.counts, data_o.old_layout.counts) and np.array_equal(data.acc_in, data_o.acc_in)
    step = engine.FrontEndStep(data)
    k0, v0 = data.k_pool.clone(), data.v_pool.clone()
    step.run()
    torch.cuda.synchronize()
    # ---- oracle chain
    src_w, src_h = synth.SOURCE_SIZE
    in_w, in_h = synth.input_size(w)
    mv_w, intra_w = pjo.project_blocks(data.blocks.view(pjo.BLOCK_DTYPE), data.cu_blocks, src_w, src_h, in_w, in_h,
                                       synth.MODEL_PATCH, w.grid_h, w.grid_w)
    res_w = rso.residual_proxy(data.cur, data.prev, data.field, 4, in_w, in_h, synth.MODEL_PATCH, w.grid_h, w.grid_w)
    assert np.array_equal(step.mv.cpu().numpy(), mv_w) and np.array_equal(step.intra.cpu().numpy(), intra_w)
    assert np.array_equal(step.res.cpu().numpy().view(np.uint32), res_w)
    keep_w, idx_w, off_w, acc_w = oc.score_compact(mv_w, res_w, intra_w, data.frame_type, data.cu_frames, data.acc_in.copy(),
                                                   w.grid_h, w.grid_w, w.group, w.tau_mv_sq, data.tau_res, True)
    assert np.array_equal(step.keep.cpu().numpy(), keep_w) and np.array_equal(step.kept_off.cpu().numpy(), off_w)
    assert np.array_equal(step.kept_idx.cpu().numpy()[: idx_w.size], idx_w)
    new_counts = np.diff(off_w).reshape(w.n_streams, w.stride)
    old = data.old_layout
    keys = ("src_slot", "dst_slot", "delta", "q_pos", "q_slot", "q_kind")
    cat = {k: [] for k in keys}
    cu_q, kv_len = [0], []
    for s in range(w.n_streams):
        pl = plo.plan_stream(old.frame_type[s].tolist(), old.counts[s].tolist(),
                             data.frame_type[s * w.stride: (s + 1) * w.stride].tolist(), new_counts[s].tolist(),
                             w.n_text, w.tokens_per_frame, old.block_table[s], data.bt_new[s])
        for k in keys:
            cat[k] += pl[k]
        cu_q.append(cu_q[-1] + len(pl["q_pos"]))
        kv_len.append(pl["kv_len"])
    n_r, n_e = len(cat["src_slot"]), len(cat["q_pos"])
    say(f"  {data.blocks.size} blocks, kept {idx_w.size} new tokens, {n_r} reused rows, {n_e} executed rows "
        f"(capacity {data.q_cap})")
    assert step.totals.cpu().tolist() == [n_r, n_e, 0, 0] and n_r == data.reuse_cap and n_e <= data.q_cap
    for k in ("src_slot", "dst_slot", "delta"):
        assert getattr(step, k)[:n_r].cpu().tolist() == cat[k], k
    for k in ("q_pos", "q_slot", "q_kind"):
        assert getattr(step, k)[:n_e].cpu().tolist() == cat[k], k
    assert step.cu_q.cpu().tolist() == cu_q and step.kv_len.cpu().tolist() == kv_len
    src, dst = np.asarray(cat["src_slot"]), np.asarray(cat["dst_slot"])
    q_slot, q_pos = np.asarray(cat["q_slot"]), np.asarray(cat["q_pos"], np.int32)
    delta = np.asarray(cat["delta"])
    layers = list(range(w.n_layers))
    k_rows, v_rows = oc.rerotate(hp.f64(k0[layers]), hp.f64(v0[layers]), src, dst, delta, w.rope_base)
    got_rows = step.k_pool.cpu()[:, torch.from_numpy(dst)].permute(1, 0, 2, 3).contiguous()
    say(f"  rerotate: {hp.check_rerotated(got_rows, k_rows, w.dtype)}")
    k_ref, v_ref = k0.clone(), v0.clone()
    for i, layer in enumerate(layers):
        k_ref[layer][torch.from_numpy(dst)] = hp.round_like(k_rows[:, i], torch.bfloat16)
        v_ref[layer][torch.from_numpy(dst)] = hp.round_like(v_rows[:, i], torch.bfloat16)
        oc.scatter(k_ref[layer].view(torch.int16).numpy(), data.k_new[layer][:n_e].view(torch.int16).numpy(), q_slot)
        oc.scatter(v_ref[layer].view(torch.int16).numpy(), data.v_new[layer][:n_e].view(torch.int16).numpy(), q_slot)
    assert torch.equal(step.v_pool.cpu().view(torch.int16), v_ref.view(torch.int16))       # values: bit-exact moves
    qs = torch.from_numpy(q_slot)
    assert torch.equal(step.k_pool.cpu()[:, qs].view(torch.int16), data.k_new[:, :n_e].view(torch.int16))
    for layer in layers:
        ref = oc.window_attn(hp.f64(data.q[layer][:n_e]), hp.f64(step.k_pool[layer]), hp.f64(step.v_pool[layer]),
                             np.asarray(cu_q, np.int32), q_pos, data.bt_new, w.n_q_heads, data.softmax_scale)
        say(f"  attention layer {layer}: {hp.check_attention(step.out[layer][:n_e].cpu(), ref, w.dtype)}")
    assert not step.out[:, n_e:].any()


FULL_WORKLOADS = [synth.CFG1, synth.CFG2, synth.CFG3P, synth.CFG3D, synth.CFG4]


@pytest.mark.parametrize("wi", range(len(FULL_WORKLOADS)))
def test_full_size_step_sampled(cs, wi):
    """The benchmark's own launch configuration at full size (the step bench.py times: refresh plan
    made on the GPU, lists padded to capacities 1/8 above the row counts); the oracle checks (a) and
    the plan completely, (c) completely, and (b), (d) on sampled rows / queries.  The queries are
    drawn by the attention call's own decomposition: at least one from every 128-row tile of every
    (stream, kv head) pair, every query head of it evaluated, plus each stream's first and last
    query, so that every work item of the launch (and every key range of a split sweep) contributes
    to a checked row; the first, a middle and the last layer are checked (the middle and last ones
    reuse the first layer's work plan).  Big tensors are drawn on the GPU by torch's generator and
    the sampled rows are copied to the host for the oracle."""
    w = FULL_WORKLOADS[wi]
    say(f"full-size step: {w.name}")
    data = engine.assemble_step(w, engine.hip_scorer, device=DEV)
    data_o = engine.assemble_step(w, hp.oracle_scorer, device="cpu", with_tensors=False)
    assert np.array_equal(data.old_layout.counts, data_o.old_layout.counts)
    assert np.array_equal(data.new_layout.counts, data_o.new_layout.counts)
    assert np.array_equal(data.new_layout.block_table, data_o.new_layout.block_table)
    say(f"  sizes: {data.info}")
    p = hp.OraclePlan(data_o)                                   # row lists from the plan oracle
    rng = np.random.default_rng(900 + wi)
    k_before = data.k_pool.clone()
    v_before = data.v_pool.clone()
    cap = lambda n: (n + n // 8 + 255) // 256 * 256
    step = engine.DeviceStep(data, reuse_cap=cap(data.info["n_reuse"]), q_cap=cap(data.info["n_q"]))
    step.run()
    torch.cuda.synchronize()
    assert step.scoring_status() == 0
    keep_w, idx_w, off_w, _ = hp.oracle_scorer(data.mv, data.sad, data.frame_type, data.cu_frames, data.acc_in,
                                               w, w.tau_mv_sq, w.tau_sad)
    assert np.array_equal(step.keep.cpu().numpy(), keep_w)
    assert np.array_equal(step.kept_off.cpu().numpy(), off_w)
    assert np.array_equal(step.kept_idx.cpu().numpy()[: idx_w.size], idx_w)
    hp.assert_device_plan(step, p)
    # (b) sampled reused rows, all layers
    n_rows = int(p.src_slot.size)
    pick = np.sort(rng.choice(n_rows, size=min(256, n_rows), replace=False))
    src = torch.from_numpy(p.src_slot[pick].astype(np.int64)).to(DEV)
    dst = torch.from_numpy(p.dst_slot[pick].astype(np.int64)).to(DEV)
    k_src = k_before[:, src].cpu()
    k_ref = np.transpose(oc.rotate(hp.f64(k_src), p.delta[pick].astype(np.float64)[None, :, None], w.rope_base),
                         (1, 0, 2, 3))
    got = step.k_pool[:, dst].cpu().permute(1, 0, 2, 3).contiguous()
    say(f"  rerotate ({pick.size} rows x {w.n_layers} layers): {hp.check_rerotated(got, k_ref, w.dtype)}")
    assert torch.equal(step.v_pool[:, dst], v_before[:, src])
    # (c) complete, bit exact (plain indexing is the definition)
    n_q = int(p.q_pos.size)
    qs = torch.from_numpy(p.q_slot.astype(np.int64)).to(DEV)
    assert torch.equal(step.k_pool[:, qs], step.k_new[:, :n_q]) and torch.equal(step.v_pool[:, qs], step.v_new[:, :n_q])
    # rows that are neither a destination nor a refresh target are untouched
    touched = torch.zeros(data.n_slots, dtype=torch.bool, device=DEV)
    touched[qs] = True
    touched[torch.from_numpy(p.dst_slot.astype(np.int64)).to(DEV)] = True
    assert torch.equal(step.k_pool[:, ~touched], k_before[:, ~touched])
    assert not step.out[:, n_q:].any()                           # rows past the executed rows are not written
    # (d) queries stratified by row tile, every head; the oracle reads the cache the method defines
    group = w.n_q_heads // w.n_kv_heads
    rows = []
    for s in range(w.n_streams):
        q0, q1 = int(p.cu_q[s]), int(p.cu_q[s + 1])
        if q1 == q0:
            continue
        rows += [q0, q1 - 1]
        n_r = (q1 - q0) * group
        for t0 in range(0, n_r, 128):
            r = int(rng.integers(t0, min(t0 + 128, n_r)))
            rows.append(q0 + r // group)
    rows = np.unique(np.asarray(rows, np.int64))
    for layer in sorted({0, w.n_layers // 2, w.n_layers - 1}):
        # cache for the oracle: reused rows re-rotated by the ORACLE (rounded), refresh rows from k_new
        s_of = np.searchsorted(p.cu_q, rows, side="right") - 1
        ref = np.zeros((rows.size, w.n_q_heads, w.head_dim))
        for s in np.unique(s_of):
            sel = rows[s_of == s]
            n_ctx = int(p.q_pos[sel].max()) + 1
            j = np.arange(n_ctx)
            slots = p.block_table[s, j // 16].astype(np.int64) * 16 + j % 16
            kk = _oracle_cache_rows(k_before[layer], step.k_new[layer], p, slots, w, rotate=True)
            vv = _oracle_cache_rows(v_before[layer], step.v_new[layer], p, slots, w, rotate=False)
            bt_local = np.arange(-(-n_ctx // 16), dtype=np.int32)[None]
            pad = bt_local.size * 16 - n_ctx
            kk = np.concatenate([kk, np.zeros((pad,) + kk.shape[1:])])
            vv = np.concatenate([vv, np.zeros((pad,) + vv.shape[1:])])
            q_sel = hp.f64(step.q[layer][torch.from_numpy(sel.astype(np.int64)).to(DEV)])
            ref[s_of == s] = oc.window_attn(q_sel, kk, vv, np.array([0, sel.size], np.int32), p.q_pos[sel],
                                            bt_local, w.n_q_heads, data.softmax_scale)
        got = step.out[layer][torch.from_numpy(rows.astype(np.int64)).to(DEV)].cpu()
        say(f"  attention layer {layer} ({rows.size} queries x {w.n_q_heads} heads): "
            f"{hp.check_attention(got, ref, w.dtype)}")


def _oracle_cache_rows(pool_before, new_rows, plan, slots, w, rotate):
    """What the oracle says the new window's cache holds at `slots` (float64 [n, Hkv, d])."""
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    n_slots = pool_before.shape[0]
    src_of = np.full(n_slots, -1, np.int64)
    src_of[plan.dst_slot] = np.arange(plan.dst_slot.size)
    new_of = np.full(n_slots, -1, np.int64)
    new_of[plan.q_slot] = np.arange(plan.q_slot.size)
    out = np.zeros((slots.size, w.n_kv_heads, w.head_dim))
    is_new = new_of[slots] >= 0
    out[is_new] = hp.f64(new_rows[torch.from_numpy(new_of[slots][is_new]).to(new_rows.device)])
    reuse = ~is_new
    assert np.all(src_of[slots][reuse] >= 0)
    r = src_of[slots][reuse]
    old = hp.f64(pool_before[torch.from_numpy(plan.src_slot[r].astype(np.int64)).to(pool_before.device)])
    if rotate:
        old = oc.rotate(old, plan.delta[r].astype(np.float64)[:, None], w.rope_base)
        old = hp.f64(hp.round_like(old, tdt))
    out[reuse] = old
    return out


def test_graph_replay_matches_eager(cs):
    """The whole step captured in a HIP graph (what bench.py times) gives the eager results on every
    replay, with eager work and synchronisations between replays.  No memset node is recorded: the
    library clears its look-back words with a kernel."""
    w = synth.small_variant(synth.CFG1, n_layers=2)
    say(f"graph replay: {w.name}, 2 layers, 3 replays")
    data = engine.assemble_step(w, engine.hip_scorer, device="cpu")
    step = engine.DeviceStep(data)
    acc0, k0, v0 = step.acc.clone(), step.k_pool.clone(), step.v_pool.clone()

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (step.keep, step.kept_off, step.kept_idx, step.acc, step.k_pool, step.v_pool, step.out)]

    def reset():
        step.acc.copy_(acc0); step.k_pool.copy_(k0); step.v_pool.copy_(v0)
        step.out.zero_(); step.keep.zero_(); step.kept_off.zero_(); step.kept_idx.zero_()

    step.run()
    eager = snapshot()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step.run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step.run()
    for rep in range(3):
        reset()
        scratch = torch.randn(1 << 20, device=DEV).sum().item()      # eager work between replays
        assert math.isfinite(scratch)
        graph.replay()
        got = snapshot()
        for i, (a, b) in enumerate(zip(eager, got)):
            assert torch.equal(a, b), f"replay {rep}: tensor {i} differs from the eager result"


def test_graph_replay_of_the_device_planned_step(cs):
    """The step with the refresh plan made on the GPU, captured in a HIP graph: every replay gives
    the eager results (plan lists, totals, cache, attention), with the plan's output arrays and the
    workspaces dirtied between replays."""
    w = synth.small_variant(synth.CFG2, n_streams=3, n_layers=2)
    say(f"graph replay, device-planned step: {w.name}, 3 streams, 2 layers, 3 replays")
    data = engine.assemble_step(w, engine.hip_scorer, device="cpu")
    n_reuse, n_q = data.info["n_reuse"], data.info["n_q"]
    step = engine.DevicePlannedStep(data, reuse_cap=n_reuse + 200, q_cap=n_q + 200)
    k0, v0 = step.k_pool.clone(), step.v_pool.clone()
    names = ("keep", "kept_off", "src_slot", "dst_slot", "delta", "q_pos", "q_slot", "q_kind", "cu_q", "kv_len",
             "totals", "new_types_out", "new_counts_out", "k_pool", "v_pool", "out")

    def snapshot():
        torch.cuda.synchronize()
        return [getattr(step, n).clone() for n in names]

    def dirty():
        step.k_pool.copy_(k0); step.v_pool.copy_(v0)
        step.out.zero_()
        for n in ("src_slot", "dst_slot", "delta", "q_pos", "q_slot", "cu_q", "kv_len", "totals", "kept_off"):
            getattr(step, n).fill_(-5)
        step.q_kind.fill_(9)
        step.ws_p.random_(0, 255)
        step.ws_a.random_(0, 255)

    step.run()
    eager = snapshot()
    assert eager[names.index("totals")].cpu().tolist() == [n_reuse, n_q, 0, 0]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        dirty()
        step.run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step.run()
    for rep in range(3):
        dirty()
        scratch = torch.randn(1 << 20, device=DEV).sum().item()      # eager work between replays
        assert math.isfinite(scratch)
        graph.replay()
        got = snapshot()
        for n, a, b in zip(names, eager, got):
            assert torch.equal(a, b), f"replay {rep}: {n} differs from the eager result"
