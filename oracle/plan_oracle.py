"""CPU oracle of the refresh plan (host logic) -- TEST INFRASTRUCTURE ONLY.

Sec. 3.4.1 ("GOP-Guided Anchor Refresh") and Sec. 3.5 of the CodecSight paper: when a window
advances, frames that stay in the window are the overlap; overlap I-frames are anchors whose
token spans are recomputed, the other overlap frames supply reused K/V (keys position-corrected
per Eq. 6), and newly arrived frames plus the text suffix are prefilled normally.

Written as plain Python loops over frames and tokens; shares nothing with the product planner.
Pinned by the worked example of the paper's KV-management figure (tests/golden/).
"""
from __future__ import annotations

FRAME_P = 0
FRAME_I = 1


def classify_frames(new_window_types, n_new):
    """Frame-level plan for a window whose last `n_new` frames have just arrived.

    new_window_types: frame types of the new window, oldest first.
    Returns three lists of window slots: (refresh anchors, reused frames, new frames).
    """
    n = len(new_window_types)
    refresh, reuse, new = [], [], []
    for slot in range(n):
        if slot >= n - n_new:
            new.append(slot)                     # newly arrived: normal prefill, whatever its type
        elif new_window_types[slot] == FRAME_I:
            refresh.append(slot)                 # overlap I-frame: anchor, recomputed
        else:
            reuse.append(slot)                   # remaining overlap: cached K/V reused
    return refresh, reuse, new


def slot_of(block_table, j, block=16):
    """Physical cache slot of window-sequence index j under a paged layout."""
    return int(block_table[j // block]) * block + j % block


def plan_stream(old_types, old_counts, new_types, new_counts, n_text, tokens_per_frame,
                old_block_table, new_block_table, block=16):
    """Token-level plan of one stream for one slide.

    old_types / old_counts: type and kept-token count of each frame of the previous window.
    new_types / new_counts: the same for the frames that just arrived (stride = len(new_types)).
    The previous window's cache holds its kept visual tokens in frame order followed by its text
    tokens; the new window's sequence is [overlap frames][new frames][text].
    Positions are dense (frame slot * tokens_per_frame + token id), so every reused token moves by
    delta = -stride * tokens_per_frame.

    Returns a dict with
      src_slot, dst_slot, delta : one entry per reused token (cache row to re-rotate / repack)
      q_pos, q_slot, q_kind     : one entry per executed token (0 anchor, 1 new frame, 2 text);
                                  q_pos is its sequence index in the new window, q_slot its slot
      kv_len                    : sequence length of the new window
    """
    stride = len(new_types)
    window = len(old_types)
    types = list(old_types[stride:]) + list(new_types)
    counts = list(old_counts[stride:]) + list(new_counts)
    refresh, reuse, new = classify_frames(types, stride)

    # first sequence index of every frame of the old window
    old_first = []
    run = 0
    for c in old_counts:
        old_first.append(run)
        run += c

    plan = dict(src_slot=[], dst_slot=[], delta=[], q_pos=[], q_slot=[], q_kind=[])
    seq = 0
    for slot in range(window):
        for i in range(counts[slot]):
            if slot in reuse:
                old_seq = old_first[slot + stride] + i
                plan["src_slot"].append(slot_of(old_block_table, old_seq, block))
                plan["dst_slot"].append(slot_of(new_block_table, seq, block))
                plan["delta"].append(-stride * tokens_per_frame)
            else:
                plan["q_pos"].append(seq)
                plan["q_slot"].append(slot_of(new_block_table, seq, block))
                plan["q_kind"].append(0 if slot in refresh else 1)
            seq += 1
    for _ in range(n_text):
        plan["q_pos"].append(seq)
        plan["q_slot"].append(slot_of(new_block_table, seq, block))
        plan["q_kind"].append(2)
        seq += 1
    plan["kv_len"] = seq
    return plan


def plan_batch(old_types, old_counts, new_types, new_counts, n_text, tokens_per_frame,
               old_block_table, new_block_table, block=16):
    """`plan_stream` for every stream of a batch, lists concatenated stream-major (Sec. 3.5: streams
    are independent; their executed rows share one variable-length launch).

    old_types / old_counts [B][W], new_types / new_counts [B][S], block tables [B][max_blocks].
    Returns a dict of Python lists: src_slot, dst_slot, delta (reused rows), q_pos, q_slot, q_kind
    (executed rows), cu_q [B+1] (first executed row of each stream) and kv_len [B].
    """
    keys = ("src_slot", "dst_slot", "delta", "q_pos", "q_slot", "q_kind")
    out = {k: [] for k in keys}
    out["cu_q"] = [0]
    out["kv_len"] = []
    for s in range(len(old_types)):
        one = plan_stream(list(old_types[s]), list(old_counts[s]), list(new_types[s]), list(new_counts[s]),
                          n_text, tokens_per_frame, old_block_table[s], new_block_table[s], block)
        for k in keys:
            out[k] += one[k]
        out["cu_q"].append(len(out["q_pos"]))
        out["kv_len"].append(one["kv_len"])
    return out
