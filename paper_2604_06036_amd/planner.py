"""Host-side refresh planner: turns frame types and kept-token counts into the row lists that the
four device calls consume.

Paper Sec. 3.4.1 (GOP-guided anchor refresh) and Sec. 3.5 (planning is separated from KV-context
preparation; a frame-aware index maps visual-token spans to physical cache slots across cache
block boundaries).  For a window that advanced by S frames:

  overlap I-frames          -> anchors: every token is recomputed (a query, written by the scatter)
  other overlap frames      -> reused: cache rows repacked into the new window's blocks with the
                               RoPE correction for the position shift
  the S new frames + text   -> prefilled normally (queries)

The window sequence is [overlap frames' kept tokens][new frames' kept tokens][text]; causality in
attention follows this sequence index.  RoPE positions are dense (frame slot * T + token id), so
every reused token moves by -S*T positions.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

FRAME_I = 1
KV_BLOCK = 16

KIND_ANCHOR = 0
KIND_NEW = 1
KIND_TEXT = 2


@dataclass
class WindowLayout:
    """What one batch of stream windows currently holds in the cache."""
    frame_type: np.ndarray    # uint8 [B, W]
    counts: np.ndarray        # int32 [B, W]  kept visual tokens per frame
    n_text: int
    block_table: np.ndarray   # int32 [B, max_blocks]

    @property
    def seq_len(self) -> np.ndarray:
        return self.counts.sum(axis=1).astype(np.int32) + np.int32(self.n_text)


@dataclass
class StepPlan:
    src_slot: np.ndarray      # int32 [n_reuse]
    dst_slot: np.ndarray      # int32 [n_reuse]
    delta: np.ndarray         # int32 [n_reuse]
    q_pos: np.ndarray         # int32 [n_q]   window-sequence index of each executed token
    q_slot: np.ndarray        # int32 [n_q]   destination cache slot of each executed token
    q_kind: np.ndarray        # uint8 [n_q]   KIND_*
    cu_q: np.ndarray          # int32 [B+1]
    kv_len: np.ndarray        # int32 [B]
    layout: WindowLayout      # the new window


def blocks_needed(seq_len) -> np.ndarray:
    return (np.asarray(seq_len, dtype=np.int64) + KV_BLOCK - 1) // KV_BLOCK


def _slots(block_row: np.ndarray, seq_idx: np.ndarray) -> np.ndarray:
    return block_row[seq_idx // KV_BLOCK].astype(np.int64) * KV_BLOCK + seq_idx % KV_BLOCK


def plan_slide(old: WindowLayout, new_types: np.ndarray, new_counts: np.ndarray,
               new_block_table: np.ndarray, tokens_per_frame: int) -> StepPlan:
    """Plan one slide for every stream of the batch.  new_types / new_counts: [B, S]."""
    n_streams, window = old.frame_type.shape
    stride = int(new_types.shape[1])
    types = np.concatenate([old.frame_type[:, stride:], new_types], axis=1).astype(np.uint8)
    counts = np.concatenate([old.counts[:, stride:], new_counts], axis=1).astype(np.int32)
    layout = WindowLayout(types, counts, old.n_text, new_block_table.astype(np.int32))

    frame_slot = np.arange(window)
    is_new = frame_slot >= window - stride
    old_start = np.concatenate([np.zeros((n_streams, 1), np.int64),
                                np.cumsum(old.counts, axis=1, dtype=np.int64)], axis=1)
    new_start = np.concatenate([np.zeros((n_streams, 1), np.int64),
                                np.cumsum(counts, axis=1, dtype=np.int64)], axis=1)

    src, dst, q_pos, q_slot, q_kind, cu_q = [], [], [], [], [], [0]
    for s in range(n_streams):
        n_vis = int(new_start[s, window])
        seq = np.arange(n_vis, dtype=np.int64)
        frame_of = np.repeat(frame_slot, counts[s])                 # window slot of each token
        within = seq - new_start[s, frame_of]
        executed = is_new[frame_of] | (types[s, frame_of] == FRAME_I)
        reused = ~executed
        # reused rows: same token, found in the old window `stride` frame slots later
        old_seq = old_start[s, frame_of[reused] + stride] + within[reused]
        src.append(_slots(old.block_table[s], old_seq))
        dst.append(_slots(new_block_table[s], seq[reused]))
        # executed rows, in sequence order, then the text suffix
        text = n_vis + np.arange(old.n_text, dtype=np.int64)
        pos = np.concatenate([seq[executed], text])
        kind = np.concatenate([np.where(is_new[frame_of[executed]], KIND_NEW, KIND_ANCHOR),
                               np.full(old.n_text, KIND_TEXT)])
        q_pos.append(pos)
        q_slot.append(_slots(new_block_table[s], pos))
        q_kind.append(kind)
        cu_q.append(cu_q[-1] + pos.shape[0])

    src_slot = np.concatenate(src).astype(np.int32)
    return StepPlan(
        src_slot=src_slot,
        dst_slot=np.concatenate(dst).astype(np.int32),
        delta=np.full(src_slot.shape, -stride * tokens_per_frame, dtype=np.int32),
        q_pos=np.concatenate(q_pos).astype(np.int32),
        q_slot=np.concatenate(q_slot).astype(np.int32),
        q_kind=np.concatenate(q_kind).astype(np.uint8),
        cu_q=np.asarray(cu_q, dtype=np.int32),
        kv_len=layout.seq_len,
        layout=layout,
    )
