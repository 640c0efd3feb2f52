"""CPU oracle for the codec-guided sliding-window prefill step (CodecSight, arXiv 2604.06036).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the HIP kernels are
checked against.  It shares no code with the GPU path and must never be imported by the product
package: only tests, the smoke check and the CPU-baseline leg of the benchmark may call it.

Everything is NumPy in float64 (integers for the mask logic).  Inputs are ordinary NumPy arrays;
bf16 data is widened to float32/float64 by the caller before it gets here, and nothing in here
rounds a result to a storage type.  Loops run over streams / frames / heads; the work inside a
loop body is the textbook formula written out once, with a matmul or an exp as a library step.

Parity pins (tests/test_oracle_pins.py, `-m "not gpu"`): every function below is pinned to
something other than itself -- closed forms, invariants, brute force over tiny inputs, a library
attention routine, and the worked refresh example of the paper's KV-management figure (for the
planner in plan_oracle.py).  No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

FRAME_P = 0
FRAME_I = 1


# --------------------------------------------------------------------------------------------
# (a) change scoring + ordered compaction      Sec. 3.3.1 (Eq. 1), Sec. 3.3.2 (Eq. 3, 4, 5),
#     "Temporal stabilization within a GOP", "Adapting sparsity to the model layout"
# --------------------------------------------------------------------------------------------
def patch_decision(mv, sad, intra, tau_mv_sq, tau_sad, use_residual):
    """Per-frame retention mask D_t(i) of one P-frame (Eq. 3-5), at patch granularity.

    mv: int array [P, 2] (dx, dy);  sad: unsigned array [P] or None;  intra: array [P] or None.
    The motion magnitude of Eq. 1 is the Euclidean norm; it is compared squared, in exact
    integers, so `V >= tau` is `dx^2 + dy^2 >= tau^2` with no rounding.
    """
    dx = mv[:, 0].astype(np.int64)
    dy = mv[:, 1].astype(np.int64)
    v_sq = dx * dx + dy * dy
    d_mv = v_sq >= np.int64(tau_mv_sq)                                   # Eq. 3
    if use_residual:
        d_res = (~d_mv) & (sad.astype(np.int64) >= np.int64(tau_sad))    # Eq. 4
    else:
        d_res = np.zeros_like(d_mv)                                      # "0 when disabled"
    d_intra = (intra != 0) if intra is not None else np.zeros_like(d_mv)
    return d_mv | d_res | d_intra                                        # Eq. 5


def tokens_from_patches(patch_mask, grid_h, grid_w, group):
    """Layout adapter: a visual token is kept if any patch of its group x group block is kept."""
    m = patch_mask.reshape(grid_h // group, group, grid_w // group, group)
    return m.any(axis=(1, 3)).reshape(-1)


def score_compact(mv, sad, intra, frame_type, cu_frames, acc_mask, grid_h, grid_w, group,
                  tau_mv_sq, tau_sad, use_residual):
    """Scoring + GOP accumulation + layout adapter + order-preserving selection.

    mv [F,P,2] int16, sad [F,P] uint32 or None, intra [F,P] uint8 or None, frame_type [F],
    cu_frames [B+1], acc_mask [B,P] uint8 or None (None = no temporal accumulation).
    Returns (keep [F,T] uint8, kept_idx int32 [n_kept], kept_off int32 [F+1], acc_out or None).
    acc_mask is not modified; the updated state is returned.
    """
    n_frames = int(frame_type.shape[0])
    n_streams = int(cu_frames.shape[0]) - 1
    n_patch = grid_h * grid_w
    n_tok = (grid_h // group) * (grid_w // group)
    keep = np.zeros((n_frames, n_tok), dtype=np.uint8)
    acc_out = None if acc_mask is None else acc_mask.astype(bool).copy()
    for s in range(n_streams):
        for f in range(int(cu_frames[s]), int(cu_frames[s + 1])):       # temporal order
            if int(frame_type[f]) == FRAME_I:
                keep[f, :] = 1                    # I-frames keep every patch
                if acc_out is not None:
                    acc_out[s, :] = False         # ... and reset the accumulation; the I-frame's
                continue                          # own full mask is not accumulated
            d = patch_decision(mv[f], None if sad is None else sad[f],
                               None if intra is None else intra[f],
                               tau_mv_sq, tau_sad, use_residual)
            if acc_out is not None:
                acc_out[s, :] |= d                # selected now or in an earlier P-frame of the GOP
                patch_mask = acc_out[s].copy()
            else:
                patch_mask = d
            assert patch_mask.shape[0] == n_patch
            keep[f, :] = tokens_from_patches(patch_mask, grid_h, grid_w, group)
    # order-preserving selection: frame-major, row-major inside the token grid
    kept_idx = np.flatnonzero(keep.reshape(-1)).astype(np.int32)
    counts = keep.sum(axis=1, dtype=np.int64)
    kept_off = np.zeros(n_frames + 1, dtype=np.int32)
    kept_off[1:] = np.cumsum(counts)
    return keep, kept_idx, kept_off, (None if acc_out is None else acc_out.astype(np.uint8))


# --------------------------------------------------------------------------------------------
# (b) position correction of reused keys       Sec. 3.4.2, Eq. 6
# --------------------------------------------------------------------------------------------
def rope_frequencies(head_dim, base):
    """theta_i = base^(-2i/d), i < d/2 (standard one-dimensional RoPE with fixed frequencies)."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    return np.power(np.float64(base), -2.0 * i / np.float64(head_dim))


def _pair_index(head_dim, style):
    half = head_dim // 2
    if style == 0:                                    # half-split: (i, i + d/2)
        return np.arange(half), np.arange(half) + half
    return 2 * np.arange(half), 2 * np.arange(half) + 1   # interleaved: (2i, 2i+1)


def rotate(x, pos, base, style=0):
    """R(pos) x for rows x [..., d] and integer (or float) positions pos broadcastable to x[..., 0].

    Used both as plain RoPE at an absolute position (R(p) k_raw) and as the correction
    R(p_new - p_old) of Eq. 6, which for 1-D RoPE is the same operator applied to the shift.
    """
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    ia, ib = _pair_index(d, style)
    ang = np.asarray(pos, dtype=np.float64)[..., None] * rope_frequencies(d, base)
    c, s = np.cos(ang), np.sin(ang)
    out = np.empty_like(x)
    out[..., ia] = x[..., ia] * c - x[..., ib] * s
    out[..., ib] = x[..., ib] * c + x[..., ia] * s
    return out


def rerotate(k_cache, v_cache, src_slot, dst_slot, delta, base, style=0):
    """Eq. 6 on a KV pool.  k_cache, v_cache: float arrays [L, n_slots, Hkv, d] (any float dtype).

    Returns (k_rows, v_rows): float64 [n_rows, L, Hkv, d], the un-rounded values that belong in
    K[l][dst_slot[r]] (or K[l][src_slot[r]] in place) and, when repacking, V[l][dst_slot[r]].
    Values are carried over unchanged (V_hat = V).  v_rows is None when dst_slot is None.
    """
    src = np.asarray(src_slot, dtype=np.int64)
    k_src = np.asarray(k_cache)[:, src].astype(np.float64)          # [L, n, Hkv, d]
    k_rows = rotate(k_src, np.asarray(delta, dtype=np.float64)[None, :, None], base, style)
    k_rows = np.transpose(k_rows, (1, 0, 2, 3))
    v_rows = None
    if dst_slot is not None:
        v_rows = np.transpose(np.asarray(v_cache)[:, src].astype(np.float64), (1, 0, 2, 3))
    return k_rows, v_rows


def rotate_axes(x, pos3, axis_of_pair, base, style=0):
    """Multidimensional RoPE (Sec. 3.4.2: each rotary dimension is corrected by the positional
    component the model maps to it).  A position is a triple (t, h, w); frequency
    pair i, with the same theta_i as 1-D RoPE, is driven by component axis_of_pair[i]:

        angle_i = pos3[..., axis_of_pair[i]] * theta_i

    x [..., d]; pos3 broadcastable to x[..., 0] + (3,); axis_of_pair int [d/2] with values 0..2.
    As with `rotate`, applied to a shift p_new - p_old it is the correction of Eq. 6, because
    rotations of one pair by different angles compose by adding the angles.
    """
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    ia, ib = _pair_index(d, style)
    axis = np.asarray(axis_of_pair, dtype=np.int64)
    assert axis.shape == (d // 2,) and axis.min() >= 0 and axis.max() <= 2
    pos_of_pair = np.asarray(pos3, dtype=np.float64)[..., axis]          # [..., d/2]
    ang = pos_of_pair * rope_frequencies(d, base)
    c, s = np.cos(ang), np.sin(ang)
    out = np.empty_like(x)
    out[..., ia] = x[..., ia] * c - x[..., ib] * s
    out[..., ib] = x[..., ib] * c + x[..., ia] * s
    return out


def rerotate_axes(k_cache, v_cache, src_slot, dst_slot, delta3, axis_of_pair, base, style=0):
    """Eq. 6 on a KV pool for multidimensional RoPE: delta3 int [n_rows, 3] is the per-row shift
    (d_t, d_h, d_w).  Same return convention as `rerotate`."""
    src = np.asarray(src_slot, dtype=np.int64)
    k_src = np.asarray(k_cache)[:, src].astype(np.float64)          # [L, n, Hkv, d]
    d3 = np.asarray(delta3, dtype=np.float64)[None, :, None, :]     # [1, n, 1, 3]
    k_rows = np.transpose(rotate_axes(k_src, d3, axis_of_pair, base, style), (1, 0, 2, 3))
    v_rows = None
    if dst_slot is not None:
        v_rows = np.transpose(np.asarray(v_cache)[:, src].astype(np.float64), (1, 0, 2, 3))
    return k_rows, v_rows


# --------------------------------------------------------------------------------------------
# (c) refresh write        Sec. 3.5: new K/V rows go straight into the destination cache
# --------------------------------------------------------------------------------------------
def scatter(cache_layer, new_rows, slot):
    """cache_layer[slot[i]] = new_rows[i] for slot[i] >= 0 (in place on the given array)."""
    for i, s in enumerate(np.asarray(slot).tolist()):
        if s >= 0:
            cache_layer[s] = new_rows[i]
    return cache_layer


# --------------------------------------------------------------------------------------------
# (d) joint prefill attention over the mixed cache          Sec. 3.5
# --------------------------------------------------------------------------------------------
def window_attn(q, k_cache_layer, v_cache_layer, cu_q, q_pos, block_table, n_q_heads,
                softmax_scale, rows=None, block=16):
    """Causal GQA attention of the executed tokens over their stream's cache.

    q [n_q, Hq, d]; k_cache_layer, v_cache_layer [n_slots, Hkv, d]; cu_q [B+1]; q_pos [n_q];
    block_table [B, max_blocks].  Query t of stream s sees cache entries j = 0..q_pos[t], entry j
    stored in slot block_table[s, j // block] * block + j % block.  Query head h reads kv head
    h // (Hq // Hkv).  `rows`: optional sorted list of query indices to evaluate (sampling for
    large cases); the result then has one row per listed query.
    Returns float64 [n_rows, Hq, d].
    """
    q = np.asarray(q)
    n_kv_heads = k_cache_layer.shape[1]
    rep = n_q_heads // n_kv_heads
    all_rows = np.arange(q.shape[0]) if rows is None else np.asarray(rows, dtype=np.int64)
    out = np.zeros((all_rows.shape[0], n_q_heads, q.shape[2]), dtype=np.float64)
    n_streams = int(cu_q.shape[0]) - 1
    for s in range(n_streams):
        sel = np.flatnonzero((all_rows >= cu_q[s]) & (all_rows < cu_q[s + 1]))
        if sel.size == 0:
            continue
        t = all_rows[sel]
        pos = np.asarray(q_pos)[t].astype(np.int64)
        n_ctx = int(pos.max()) + 1                      # cache entries any of these queries sees
        j = np.arange(n_ctx)
        slots = block_table[s, j // block].astype(np.int64) * block + j % block
        visible = j[None, :] <= pos[:, None]            # causal rule by window-sequence index
        for h in range(n_q_heads):
            g = h // rep
            kk = k_cache_layer[slots, g].astype(np.float64)       # [n_ctx, d]
            vv = v_cache_layer[slots, g].astype(np.float64)
            sc = np.float64(softmax_scale) * (q[t, h].astype(np.float64) @ kk.T)
            sc = np.where(visible, sc, -np.inf)
            p = np.exp(sc - sc.max(axis=1, keepdims=True))
            out[sel, h] = (p @ vv) / p.sum(axis=1, keepdims=True)
    return out


def full_causal(q, k, v, softmax_scale):
    """Plain causal attention of a whole sequence: q [n, Hq, d], k, v [n, Hkv, d] -> [n, Hq, d].

    The nothing-pruned / nothing-reused reference: every token is a query at its own index.
    """
    n, n_q_heads, _ = q.shape
    rep = n_q_heads // k.shape[1]
    out = np.zeros(q.shape, dtype=np.float64)
    visible = np.tril(np.ones((n, n), dtype=bool))
    for h in range(n_q_heads):
        g = h // rep
        sc = np.float64(softmax_scale) * (q[:, h].astype(np.float64) @ k[:, g].astype(np.float64).T)
        sc = np.where(visible, sc, -np.inf)
        p = np.exp(sc - sc.max(axis=1, keepdims=True))
        out[:, h] = (p @ v[:, g].astype(np.float64)) / p.sum(axis=1, keepdims=True)
    return out
