"""cs_score_compact_noalloc (the entry point that allocates nothing) against cs_score_compact,
through the C ABI, on two calls in a row, the second with a smaller input (needs an MI355X)."""
import sys

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _inputs(rng, n_streams, frames_per_stream, gh, gw):
    counts = np.full(n_streams, frames_per_stream, np.int32)
    cu = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    n_frames, n_patch = int(cu[-1]), gh * gw
    mv = np.rint(rng.normal(0, 6, size=(n_frames, n_patch, 2))).astype(np.int16)
    sad = rng.integers(0, 1200, size=(n_frames, n_patch), dtype=np.uint32)
    intra = (rng.random((n_frames, n_patch)) < 0.02).astype(np.uint8)
    ft = (rng.random(n_frames) < 0.2).astype(np.uint8)
    acc = (rng.random((n_streams, n_patch)) < 0.1).astype(np.uint8)
    return mv, sad, intra, ft, cu, acc


def _run(cs, ins, gh, gw, group, static):
    mv, sad, intra, ft, cu, acc = ins
    n_frames, n_streams = int(ft.shape[0]), int(cu.shape[0]) - 1
    t_per = (gh // group) * (gw // group)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    d_acc = d(acc)
    keep = torch.full((n_frames, t_per), 9, dtype=torch.uint8, device=DEV)
    idx = torch.full((n_frames * t_per,), -7, dtype=torch.int32, device=DEV)
    off = torch.full((n_frames + 1,), -7, dtype=torch.int32, device=DEV)
    args = (d(mv), d(sad.view(np.int32)), d(intra), d(ft), d(cu), d_acc, n_streams, n_frames, gh, gw, group, 17, 401,
            True, keep, idx, off)
    if static:
        cs.cs_score_compact_noalloc(*args)
    else:
        nbytes = cs.cs_score_compact_workspace(n_streams, n_frames, gh, gw, group)
        ws = torch.randint(0, 255, (max(8, nbytes),), dtype=torch.uint8, device=DEV)
        cs.cs_score_compact(*args, ws, nbytes)
    torch.cuda.synchronize()
    return [t.cpu().numpy() for t in (keep, idx, off, d_acc)]


def test_noalloc_scoring_equals_the_workspace_call_twice_in_a_row():
    from paper_2604_06036_amd import binding as cs
    rng = np.random.default_rng(20260)
    # many tiles (look-back words in use), then a smaller batch, then one that fits a single tile
    cases = [(300, 3, 16, 16, 1), (37, 2, 16, 16, 1), (3, 4, 12, 8, 2), (64, 1, 16, 16, 1)]
    for n_streams, fps, gh, gw, group in cases:
        print(f"[case] noalloc scoring: streams={n_streams} frames/stream={fps} grid={gh}x{gw} group={group}", flush=True)
        sys.stdout.flush()
        ins = _inputs(rng, n_streams, fps, gh, gw)
        want = _run(cs, ins, gh, gw, group, static=False)
        got = _run(cs, ins, gh, gw, group, static=True)
        for name, a, b in zip(("keep", "kept_idx", "kept_off", "acc"), want, got):
            assert np.array_equal(a, b), name


def test_noalloc_scoring_rejects_batches_beyond_its_scratch():
    from paper_2604_06036_amd import binding as cs
    print("[case] noalloc scoring: 4097 streams is beyond the static scratch", flush=True)
    z = torch.zeros((16,), dtype=torch.int32, device=DEV)
    with pytest.raises(cs.CodecSightError) as exc:
        cs.lib()                                  # make sure the library is loaded
        rc = cs.lib().cs_score_compact_noalloc(None, None, None, None, None, None, 4097, 4097, 16, 16, 1, 0, 0, 0,
                                               None, None, None, None)
        cs._check("cs_score_compact_noalloc", rc)
    assert exc.value.code == cs.CS_EUNSUPPORTED
