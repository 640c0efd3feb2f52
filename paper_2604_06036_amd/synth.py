"""Seeded synthetic inputs shaped like the paper's streaming-video workloads.

This module only draws random inputs (codec metadata, frame-type schedules, block tables,
Q/K/V tensors).  It applies none of the method's arithmetic -- no thresholds, no masks, no
rotations, no attention -- so it can feed both the HIP path and the CPU oracle.

Geometry follows the paper: 448x448 frames give a 16x16 grid of merged visual tokens, I+P GOPs,
one window per stride, many independent streams.  The videos, questions and model weights behind
the paper's evaluation are not available here; these streams stand in for them.

Recipe (per stream s of workload w, rng = default_rng(SeedSequence([0xC0DEC, w.seed_id, s]))):
  frame types  I-frames every `gop` frames, phase chosen so that slot `i_slot` of the NEW window
               is an I-frame; history = 2*max(gop) warm-up frames + the old window + the stride.
  moving blobs discs on the patch grid, radii U[1.5, 3.5] patches scaled by one bisected factor
               so that the rasterised area is within 2 p.p. of the stream's moving fraction;
               centres random-walk N(0, 0.5^2) patches per frame, reflected at the borders.
  MV           int16 quarter-pel components: round(N(0,1)) outside blobs, round(N(0,24)) inside
               (24 is the standard deviation).
  SAD          uint32 round(Gamma(k=2, theta=50)), multiplied by 10 inside blobs.
  I-frames     carry zero metadata.
  Q/K/V, cache N(0,1), float32 then cast to the workload dtype.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Tuple

import numpy as np

FRAME_P = 0
FRAME_I = 1
KV_BLOCK = 16


@dataclass(frozen=True)
class Workload:
    name: str
    seed_id: int
    n_streams: int
    dtype: str                      # "f32" | "bf16"
    window: int                     # frames per window (W)
    stride: int                     # new frames per slide (S)
    grid_h: int
    grid_w: int
    n_text: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rope_base: float
    n_layers: int
    gop_choices: Tuple[int, ...]
    i_slot: int                     # I-frame slot in the new window; -1 = uniform over the GOP
    moving: Tuple[str, float, float]  # ("const", m, _) | ("uniform", lo, hi) | ("beta", a, b)
    group: int = 1
    tau_mv_sq: int = 17             # |MV| > 4 quarter-pel  <=>  dx^2+dy^2 >= 17
    tau_sad: int = 401              # SAD > 400
    use_residual: bool = True
    dense_history: bool = False     # overlap frames cached unpruned (literal "dense rows" reading)
    shuffle_blocks: bool = True

    @property
    def patches(self) -> int:
        return self.grid_h * self.grid_w

    @property
    def tokens_per_frame(self) -> int:
        return (self.grid_h // self.group) * (self.grid_w // self.group)

    @property
    def history(self) -> int:
        return 2 * max(self.gop_choices) + self.window + self.stride

    @property
    def position_shift(self) -> int:
        return -self.stride * self.tokens_per_frame


# The five configurations of the benchmark definition (3p / 3d are the two readings of the
# long-window case: cache pruned as the method would leave it, or holding dense rows).
CFG0 = Workload("cfg0_tiny_f32", 0, 1, "f32", 4, 1, 16, 16, 16, 2, 1, 64, 1e4, 1,
                (4,), 0, ("const", 0.20, 0.0), shuffle_blocks=False)
CFG1 = Workload("cfg1_qwen7b_1stream", 1, 1, "bf16", 8, 1, 16, 16, 64, 28, 4, 128, 1e6, 28,
                (8,), 0, ("const", 0.25, 0.0), shuffle_blocks=False)
CFG2 = Workload("cfg2_qwen7b_32streams", 2, 32, "bf16", 8, 1, 16, 16, 64, 28, 4, 128, 1e6, 28,
                (8,), -1, ("uniform", 0.05, 0.40))
CFG3P = Workload("cfg3p_longwindow_pruned", 3, 1, "bf16", 16, 2, 26, 46, 128, 28, 4, 128, 1e6, 28,
                 (16,), 0, ("const", 0.15, 0.0), shuffle_blocks=False)
CFG3D = replace(CFG3P, name="cfg3d_longwindow_dense", dense_history=True)
CFG4 = Workload("cfg4_internlm7b_64streams", 4, 64, "bf16", 8, 1, 16, 16, 32, 32, 8, 128, 1e6, 32,
                (4, 8, 16), -1, ("beta", 2.0, 8.0))

WORKLOADS = {w.name: w for w in (CFG0, CFG1, CFG2, CFG3P, CFG3D, CFG4)}


def small_variant(w: Workload, n_streams: int | None = None, n_layers: int | None = None) -> Workload:
    """Same shapes with fewer streams / layers (parity cases the CPU oracle finishes quickly)."""
    return replace(w, n_streams=n_streams or w.n_streams, n_layers=n_layers or w.n_layers)


def _rng(w: Workload, *tag: int) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([0xC0DEC, w.seed_id, *tag]))


def _reflect(x: np.ndarray, hi: float) -> np.ndarray:
    x = np.abs(x)
    return np.where(x > hi, 2.0 * hi - x, x)


def _blob_mask(cy, cx, rad, grid_h, grid_w) -> np.ndarray:
    """[n_frames, P] bool: patch centre inside any disc.  cy, cx: [n_frames, n_blobs]."""
    yy, xx = np.meshgrid(np.arange(grid_h) + 0.5, np.arange(grid_w) + 0.5, indexing="ij")
    yy = yy.reshape(1, 1, -1)
    xx = xx.reshape(1, 1, -1)
    d2 = (yy - cy[..., None]) ** 2 + (xx - cx[..., None]) ** 2
    return (d2 <= (rad[None, :, None] ** 2)).any(axis=1)


@dataclass
class StreamMeta:
    gop: int
    moving_target: float
    frame_type: np.ndarray   # uint8 [H]
    mv: np.ndarray           # int16 [H, P, 2]
    sad: np.ndarray          # uint32 [H, P]
    blob: np.ndarray         # bool [H, P] (where the generator put motion; informational)


def stream_metadata(w: Workload, s: int) -> StreamMeta:
    """Codec metadata of the whole history of stream s (oldest frame first)."""
    rng = _rng(w, s)
    n_hist, n_patch = w.history, w.patches
    gop = int(rng.choice(np.asarray(w.gop_choices)))
    i_slot = w.i_slot if w.i_slot >= 0 else int(rng.integers(0, gop))
    kind, a, b = w.moving
    if kind == "const":
        target = a
    elif kind == "uniform":
        target = float(rng.uniform(a, b))
    else:
        target = float(rng.beta(a, b))

    # frame types: the new window occupies history slots [H-W, H); its slot i_slot is an I-frame
    anchor = n_hist - w.window + i_slot
    idx = np.arange(n_hist)
    frame_type = np.where((idx - anchor) % gop == 0, FRAME_I, FRAME_P).astype(np.uint8)

    # blobs
    mean_area = np.pi * 2.5 ** 2
    n_blobs = max(1, int(round(target * n_patch / mean_area)))
    rad0 = rng.uniform(1.5, 3.5, size=n_blobs)
    cy0 = rng.uniform(0.0, w.grid_h, size=n_blobs)
    cx0 = rng.uniform(0.0, w.grid_w, size=n_blobs)
    lo, hi = 0.05, 6.0
    for _ in range(40):                      # bisect one common radius scale on the first frame
        mid = 0.5 * (lo + hi)
        frac = _blob_mask(cy0[None], cx0[None], rad0 * mid, w.grid_h, w.grid_w).mean()
        if frac > target:
            hi = mid
        else:
            lo = mid
    rad = rad0 * 0.5 * (lo + hi)
    steps = rng.normal(0.0, 0.5, size=(n_hist, n_blobs, 2))
    steps[0] = 0.0
    cy = _reflect(cy0[None] + np.cumsum(steps[..., 0], axis=0), float(w.grid_h))
    cx = _reflect(cx0[None] + np.cumsum(steps[..., 1], axis=0), float(w.grid_w))
    blob = _blob_mask(cy, cx, rad, w.grid_h, w.grid_w)

    sigma = np.where(blob, 24.0, 1.0)[..., None]
    mv = np.rint(rng.normal(0.0, 1.0, size=(n_hist, n_patch, 2)) * sigma)
    mv = np.clip(mv, -32768, 32767).astype(np.int16)
    sad = np.rint(rng.gamma(2.0, 50.0, size=(n_hist, n_patch)) * np.where(blob, 10.0, 1.0))
    sad = sad.astype(np.uint32)
    is_i = frame_type == FRAME_I
    mv[is_i] = 0
    sad[is_i] = 0
    return StreamMeta(gop, target, frame_type, mv, sad, blob)


@dataclass
class BatchMeta:
    """History of all streams, stream-major: frame f of stream s is row s*H + f."""
    workload: Workload
    frame_type: np.ndarray   # uint8 [B*H]
    mv: np.ndarray           # int16 [B*H, P, 2]
    sad: np.ndarray          # uint32 [B*H, P]
    gop: np.ndarray          # int32 [B]
    moving_target: np.ndarray

    def rows(self, first: int, count: int) -> np.ndarray:
        """Row indices of history frames [first, first+count) of every stream, stream-major."""
        h = self.workload.history
        return (np.arange(self.workload.n_streams)[:, None] * h + first + np.arange(count)[None]).reshape(-1)


def batch_metadata(w: Workload) -> BatchMeta:
    metas = [stream_metadata(w, s) for s in range(w.n_streams)]
    return BatchMeta(
        w,
        np.concatenate([m.frame_type for m in metas]),
        np.concatenate([m.mv for m in metas]),
        np.concatenate([m.sad for m in metas]),
        np.asarray([m.gop for m in metas], dtype=np.int32),
        np.asarray([m.moving_target for m in metas]),
    )


# 16-byte coding-block record of the block-to-patch projection (layout of cs_block in the C header)
BLOCK_DTYPE = np.dtype([("x", "<u2"), ("y", "<u2"), ("w", "<u2"), ("h", "<u2"),
                        ("dx", "<i2"), ("dy", "<i2"), ("flags", "<u4")])
MODEL_PATCH = 28             # input pixels per patch-grid cell (14-pixel ViT patches merged 2 x 2)
SOURCE_SIZE = (1920, 1080)   # decoded stream resolution (coded in 16 x 16 macroblocks: 120 x 68)

# macroblock partitions (offset x, offset y, width, height): one 16x16, two 16x8, two 8x16, four 8x8
_PARTITIONS = (
    ((0, 0, 16, 16),),
    ((0, 0, 16, 8), (0, 8, 16, 8)),
    ((0, 0, 8, 16), (8, 0, 8, 16)),
    ((0, 0, 8, 8), (8, 0, 8, 8), (0, 8, 8, 8), (8, 8, 8, 8)),
)
# partition mix of a P-frame's macroblocks (last entry: intra-coded), in still and in moving regions
_PARTITION_P_STILL = (0.70, 0.08, 0.08, 0.138, 0.002)
_PARTITION_P_MOVING = (0.40, 0.12, 0.12, 0.31, 0.05)


def input_size(w: Workload) -> Tuple[int, int]:
    """(width, height) of the preprocessed model input whose patch grid the workload names."""
    return w.grid_w * MODEL_PATCH, w.grid_h * MODEL_PATCH


def block_frames(w: Workload, frame_type: np.ndarray, blob: np.ndarray, tag: int = 0):
    """Per-block decoder output for a batch of frames, H.264-like: the source frame is tiled by
    16 x 16 macroblocks (the last row sticks out of a 1080-line frame), each split into one, two or
    four inter partitions with a vector of their own, or intra-coded (finer partitions and intra
    macroblocks are more frequent where the scene moves); I-frames are all intra.
    Vectors are drawn like the per-patch metadata: N(0, 24^2) where the block's centre falls on a
    moving patch (`blob` [F, P] bool), N(0, 1) elsewhere, rounded to int16.
    Returns (blocks [n] BLOCK_DTYPE, macroblock raster order, partitions in order; cu_blocks [F+1])."""
    rng = _rng(w, 0xB10C5, tag)
    src_w, src_h = SOURCE_SIZE
    mb_w, mb_h = (src_w + 15) // 16, (src_h + 15) // 16
    n_mb = mb_w * mb_h
    mb_x = (np.arange(n_mb) % mb_w) * 16
    mb_y = (np.arange(n_mb) // mb_w) * 16
    out, cu = [], [0]
    for f in range(int(frame_type.shape[0])):
        mcx = np.minimum((mb_x + 8.0) * w.grid_w / src_w, w.grid_w - 1).astype(np.int64)
        mcy = np.minimum((mb_y + 8.0) * w.grid_h / src_h, w.grid_h - 1).astype(np.int64)
        kind = np.where(blob[f, mcy * w.grid_w + mcx], rng.choice(5, size=n_mb, p=_PARTITION_P_MOVING),
                        rng.choice(5, size=n_mb, p=_PARTITION_P_STILL))
        if frame_type[f] == FRAME_I:
            kind = np.full(n_mb, 4)
        parts, order = [], []
        for k in range(5):
            mbs = np.flatnonzero(kind == k)
            for j, (ox, oy, pw, ph) in enumerate(_PARTITIONS[k] if k < 4 else _PARTITIONS[0]):
                b = np.zeros(mbs.size, BLOCK_DTYPE)
                b["x"], b["y"], b["w"], b["h"] = mb_x[mbs] + ox, mb_y[mbs] + oy, pw, ph
                b["flags"] = 1 if k == 4 else 0
                parts.append(b)
                order.append(mbs * 4 + j)
        b = np.concatenate(parts)[np.argsort(np.concatenate(order), kind="stable")]
        # which patch the block's centre falls on (only to place the motion, no part of the method)
        cx = np.minimum((b["x"] + b["w"] / 2.0) * w.grid_w / src_w, w.grid_w - 1).astype(np.int64)
        cy = np.minimum((b["y"] + b["h"] / 2.0) * w.grid_h / src_h, w.grid_h - 1).astype(np.int64)
        sigma = np.where(blob[f, cy * w.grid_w + cx], 24.0, 1.0)
        vec = np.clip(np.rint(rng.normal(0.0, 1.0, size=(b.size, 2)) * sigma[:, None]), -32768, 32767)
        inter = b["flags"] == 0
        b["dx"][inter], b["dy"][inter] = vec[inter, 0], vec[inter, 1]
        out.append(b)
        cu.append(cu[-1] + b.size)
    return np.concatenate(out) if out else np.zeros(0, BLOCK_DTYPE), np.asarray(cu, np.int32)


def motion_field(blocks: np.ndarray, cu_blocks: np.ndarray, cell: int = 4) -> np.ndarray:
    """The block lists of `block_frames` rasterised to a regular field of cell x cell pixel cells:
    int16 [F, ceil(H/cell), ceil(W/cell), 2]; intra blocks leave (0, 0).  Pure re-formatting."""
    src_w, src_h = SOURCE_SIZE
    n_frames = int(cu_blocks.shape[0]) - 1
    field = np.zeros((n_frames, -(-src_h // cell), -(-src_w // cell), 2), np.int16)
    for f in range(n_frames):
        b = blocks[cu_blocks[f]:cu_blocks[f + 1]]
        b = b[b["flags"] == 0]
        for size in np.unique(np.stack([b["w"], b["h"]], axis=1), axis=0):
            sel = b[(b["w"] == size[0]) & (b["h"] == size[1])]
            for oy in range(0, int(size[1]), cell):
                for ox in range(0, int(size[0]), cell):
                    cy, cx = (sel["y"] + oy) // cell, (sel["x"] + ox) // cell
                    ok = (cy < field.shape[1]) & (cx < field.shape[2])
                    field[f, cy[ok], cx[ok], 0] = sel["dx"][ok]
                    field[f, cy[ok], cx[ok], 1] = sel["dy"][ok]
    return field


def decoded_frames(w: Workload, n_frames: int, blob: np.ndarray, tag: int = 0):
    """(cur, prev) uint8 [F, 1080, 1920] luma planes: prev is a smooth random texture; cur repeats
    it with sensor noise (sigma 1.5 grey levels), shows it displaced by (3, -2) pixels where the
    scene moves (`blob` [F, P] bool on the patch grid) and 30 grey levels brighter on a few discs
    that do not move (appearance change without motion: what residual rescue is for)."""
    rng = _rng(w, 0xF4A3E, tag)
    src_w, src_h = SOURCE_SIZE
    cur = np.empty((n_frames, src_h, src_w), np.uint8)
    prev = np.empty_like(cur)
    yy, xx = np.meshgrid(np.arange(src_h), np.arange(src_w), indexing="ij")
    py = np.minimum(yy * w.grid_h // src_h, w.grid_h - 1)
    px = np.minimum(xx * w.grid_w // src_w, w.grid_w - 1)
    for f in range(n_frames):
        coarse = rng.integers(40, 200, size=(src_h // 8 + 1, src_w // 8 + 1)).astype(np.float32)
        tex = np.kron(coarse, np.ones((8, 8), np.float32))[:src_h, :src_w] + rng.normal(0.0, 6.0, size=(src_h, src_w))
        p = np.clip(np.rint(tex), 0, 255)
        moving = blob[f].reshape(w.grid_h, w.grid_w)[py, px]
        c = np.where(moving, np.roll(p, shift=(-2, 3), axis=(0, 1)), p) + rng.normal(0.0, 1.5, size=p.shape)
        for _ in range(3):
            cy, cx, rad = rng.uniform(0, src_h), rng.uniform(0, src_w), rng.uniform(40, 120)
            c = c + 30.0 * ((yy - cy) ** 2 + (xx - cx) ** 2 <= rad * rad)
        prev[f] = p.astype(np.uint8)
        cur[f] = np.clip(np.rint(c), 0, 255).astype(np.uint8)
    return cur, prev


def block_ids(w: Workload, n_blocks_needed: int, tag: int = 0) -> np.ndarray:
    """A pool of `n_blocks_needed` distinct physical block ids: shuffled, or 0..n-1 in order."""
    ids = np.arange(n_blocks_needed, dtype=np.int32)
    if w.shuffle_blocks:
        _rng(w, 0x0B10C, tag).shuffle(ids)
    return ids


def normal_tensor(w: Workload, tag: Tuple[int, ...], shape, device="cpu"):
    """N(0,1) tensor in the workload dtype, drawn in float32 then cast.  Returns a torch tensor.

    The seed depends on (workload, tag) only; CPU and GPU generators give different streams, so
    a test that compares against the oracle draws on the CPU and copies.
    """
    import torch
    seed = int(np.random.SeedSequence([0xC0DEC, w.seed_id, 0x7E50, *tag]).generate_state(1)[0])
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    x = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
    return x if w.dtype == "f32" else x.to(torch.bfloat16)
