"""Drives one slide step of a batch of streams through the device calls.

`assemble_step` builds everything a step needs from a synthetic workload (history scoring to get
the cached window's token layout, the step's own scoring, block tables and the Q/K/V tensors);
`DeviceStep` holds those inputs on the GPU and issues the calls in the order the method
prescribes: score+compact, refresh plan, re-rotate (all layers), then per layer refresh write
followed by attention (paper Sec. 3.5: planning first, KV-context preparation next, joint prefill
last).  The refresh plan is made on the GPU (cs_plan_refresh) and nothing passes through the host
between the calls; the NumPy planner in `planner.py` is a cross-check for tests and comparison
runs (`DeviceStep(..., host_plan=True)`), never part of the default route.

The scoring function is a parameter so that the same assembly can be driven by the HIP kernels
(`hip_scorer`, the product path) or, in tests, by the CPU oracle; nothing here falls back to a CPU
implementation on its own.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Callable, Optional

import numpy as np

from . import planner, synth


# scorer(mv, sad, frame_type, cu_frames, acc, workload, tau_mv_sq, tau_sad) ->
#     (keep [F,T] uint8, kept_idx int32, kept_off int32 [F+1], acc_out [B,P] uint8)
Scorer = Callable[..., tuple]


def hip_scorer(mv, sad, frame_type, cu_frames, acc, w: synth.Workload, tau_mv_sq: int, tau_sad: int):
    """cs_score_compact on NumPy inputs (copies in, copies out).  Product path: HIP only."""
    import torch
    from . import binding as cs
    dev = torch.device("cuda")
    n_frames, n_streams = int(frame_type.shape[0]), int(cu_frames.shape[0]) - 1
    t_per = w.tokens_per_frame
    d_mv = torch.from_numpy(mv).to(dev)
    d_sad = torch.from_numpy(sad.view(np.int32)).to(dev) if w.use_residual else None
    d_ft = torch.from_numpy(frame_type).to(dev)
    d_cu = torch.from_numpy(cu_frames).to(dev)
    d_acc = torch.from_numpy(acc).to(dev) if acc is not None else None
    keep = torch.empty((n_frames, t_per), dtype=torch.uint8, device=dev)
    idx = torch.empty((max(1, n_frames * t_per),), dtype=torch.int32, device=dev)
    off = torch.empty((n_frames + 1,), dtype=torch.int32, device=dev)
    ws_bytes = cs.cs_score_compact_workspace(n_streams, n_frames, w.grid_h, w.grid_w, w.group)
    ws = torch.empty((max(8, ws_bytes),), dtype=torch.uint8, device=dev)
    cs.cs_score_compact(d_mv, d_sad, None, d_ft, d_cu, d_acc, n_streams, n_frames, w.grid_h, w.grid_w,
                        w.group, tau_mv_sq, tau_sad, w.use_residual, keep, idx, off, ws, ws_bytes)
    torch.cuda.synchronize()
    off_h = off.cpu().numpy()
    return (keep.cpu().numpy(), idx[: int(off_h[-1])].cpu().numpy(), off_h,
            None if d_acc is None else d_acc.cpu().numpy())


@dataclass
class StepData:
    """Inputs of one slide step.  Small arrays are NumPy on the host; big tensors are torch."""
    workload: synth.Workload
    # (a) the S new frames of every stream, stream-major
    mv: np.ndarray
    sad: np.ndarray
    frame_type: np.ndarray
    cu_frames: np.ndarray
    acc_in: np.ndarray                 # accumulated mask carried in from the history
    # layouts: the cached window, and the new window's frame types / kept counts / block table
    old_layout: planner.WindowLayout
    new_layout: planner.WindowLayout
    n_slots: int
    # tensors (torch): pool [L, n_slots, Hkv, d]; q [L, n_q, Hq, d]; k_new, v_new [L, n_q, Hkv, d]
    k_pool: object = None
    v_pool: object = None
    q: object = None
    k_new: object = None
    v_new: object = None
    softmax_scale: float = 0.0
    info: dict = field(default_factory=dict)
    _plan: object = None

    @property
    def plan(self) -> planner.StepPlan:
        """The step's row lists as the host planner makes them (built on first use): the
        cross-check of cs_plan_refresh in tests and the lists of a `host_plan=True` step."""
        if self._plan is None:
            w = self.workload
            new = self.new_layout
            self._plan = planner.plan_slide(self.old_layout, new.frame_type[:, w.window - w.stride:],
                                            new.counts[:, w.window - w.stride:], new.block_table,
                                            w.tokens_per_frame)
        return self._plan


def assemble_step(w: synth.Workload, scorer: Scorer, device="cpu", with_tensors: bool = True) -> StepData:
    """History -> cached window layout -> this step's scoring -> block tables -> refresh plan."""
    meta = synth.batch_metadata(w)
    n_streams, hist, stride, window = w.n_streams, w.history, w.stride, w.window
    t_per = w.tokens_per_frame

    # 1. history (everything before the new frames), accumulated mask starting from zero
    past = hist - stride
    rows = meta.rows(0, past)
    cu = (np.arange(n_streams + 1) * past).astype(np.int32)
    acc0 = np.zeros((n_streams, w.patches), np.uint8)
    keep_h, _, off_h, acc_h = scorer(meta.mv[rows], meta.sad[rows], meta.frame_type[rows], cu, acc0, w,
                                     w.tau_mv_sq, w.tau_sad)
    counts_h = np.diff(off_h).reshape(n_streams, past)
    old_counts = counts_h[:, past - window:].astype(np.int32)
    if w.dense_history:
        old_counts = np.full_like(old_counts, t_per)          # cache holds unpruned rows
    old_types = meta.frame_type.reshape(n_streams, hist)[:, past - window: past]

    # 2. this step: the S new frames of every stream
    rows_new = meta.rows(past, stride)
    cu_new = (np.arange(n_streams + 1) * stride).astype(np.int32)
    keep_n, _, off_n, _ = scorer(meta.mv[rows_new], meta.sad[rows_new], meta.frame_type[rows_new], cu_new,
                                 acc_h.copy(), w, w.tau_mv_sq, w.tau_sad)
    new_counts = np.diff(off_n).reshape(n_streams, stride).astype(np.int32)
    new_types = meta.frame_type[rows_new].reshape(n_streams, stride)

    # 3. block tables: old and new windows draw distinct blocks from one pool
    old_len = old_counts.sum(axis=1) + w.n_text
    new_len = old_counts[:, stride:].sum(axis=1) + new_counts.sum(axis=1) + w.n_text
    nb_old, nb_new = planner.blocks_needed(old_len), planner.blocks_needed(new_len)
    ids = synth.block_ids(w, int(nb_old.sum() + nb_new.sum()))
    max_blocks = int(max(nb_old.max(), nb_new.max()))
    bt_old = np.zeros((n_streams, max_blocks), np.int32)
    bt_new = np.zeros((n_streams, max_blocks), np.int32)
    at = 0
    for s in range(n_streams):
        bt_old[s, : nb_old[s]] = ids[at: at + nb_old[s]]
        at += int(nb_old[s])
        bt_new[s, : nb_new[s]] = ids[at: at + nb_new[s]]
        at += int(nb_new[s])
    n_slots = int(ids.shape[0]) * synth.KV_BLOCK

    # 4. the two window layouts; the step's sizes follow from the counts alone (reused rows = kept
    #    tokens of the overlap's P-frames, executed rows = overlap I-frames + new frames + text)
    old_layout = planner.WindowLayout(old_types.astype(np.uint8), old_counts, w.n_text, bt_old)
    new_layout = planner.WindowLayout(np.concatenate([old_types[:, stride:], new_types], axis=1).astype(np.uint8),
                                      np.concatenate([old_counts[:, stride:], new_counts], axis=1).astype(np.int32),
                                      w.n_text, bt_new)
    data = StepData(w, meta.mv[rows_new], meta.sad[rows_new], meta.frame_type[rows_new], cu_new, acc_h,
                    old_layout, new_layout, n_slots, softmax_scale=1.0 / math.sqrt(w.head_dim))
    overlap_t, overlap_c = old_types[:, stride:], old_counts[:, stride:]
    n_reuse = int(overlap_c[overlap_t != synth.FRAME_I].sum())
    n_q = int(overlap_c[overlap_t == synth.FRAME_I].sum() + new_counts.sum() + n_streams * w.n_text)
    vis = float(new_len.sum())
    data.info = dict(n_q=n_q, n_reuse=n_reuse, kv_len_total=int(vis), n_slots=n_slots,
                     kept_new=int(new_counts.sum()), reused_fraction=float(n_reuse) / max(1.0, vis))
    if with_tensors:
        shape_pool = (w.n_layers, n_slots, w.n_kv_heads, w.head_dim)
        data.k_pool = synth.normal_tensor(w, (1,), shape_pool, device)
        data.v_pool = synth.normal_tensor(w, (2,), shape_pool, device)
        data.q = synth.normal_tensor(w, (3,), (w.n_layers, n_q, w.n_q_heads, w.head_dim), device)
        data.k_new = synth.normal_tensor(w, (4,), (w.n_layers, n_q, w.n_kv_heads, w.head_dim), device)
        data.v_new = synth.normal_tensor(w, (5,), (w.n_layers, n_q, w.n_kv_heads, w.head_dim), device)
    return data


OVERLAP_MIN_BYTES = 1 << 30     # bytes the position correction moves per step from which it runs beside the layer loop


class DeviceStep:
    """A step resident on the GPU; each method enqueues exactly one C-ABI call.

    The row lists of (b), (c), (d) are written by cs_plan_refresh from the offsets the scoring call
    leaves in device memory: no list, count or offset passes through the host between the calls.
    They are sized to capacities the caller budgets (`reuse_cap`, `q_cap`; default: the step's own
    row counts); the consumers are launched over the capacities and skip the padding.
    `host_plan=True` uploads the NumPy planner's lists instead and `run` skips the planning call
    (tests and comparison runs)."""

    def __init__(self, data: StepData, reuse_cap: Optional[int] = None, q_cap: Optional[int] = None,
                 host_plan: bool = False, fused: bool = False, overlap: Optional[bool] = None,
                 layers_per_rerotate: int = 4):
        import torch
        from . import binding as cs
        self.cs = cs
        self.data = data
        self.host_plan = host_plan
        self.fused = fused             # refresh write inside the attention launch (cs_refresh_prefill_attn)
        # overlap: the position correction runs on a second stream, a few layers per call, while the
        # layer loop proceeds; a layer's attention waits for the call that covers its layer
        # (decided below, once the capacities are known; None = by the size of the correction's traffic)
        self.overlap = overlap
        self.layers_per_rerotate = max(1, int(layers_per_rerotate))
        w = data.workload
        dev = torch.device("cuda")
        self.dev = dev
        to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        i32 = lambda n, fill: torch.full((max(1, n),), fill, dtype=torch.int32, device=dev)
        self.dtype = cs.CS_BF16 if w.dtype == "bf16" else cs.CS_F32
        # (a)
        self.mv = to(data.mv)
        self.sad = to(data.sad.view(np.int32)) if w.use_residual else None
        self.frame_type = to(data.frame_type)
        self.cu_frames = to(data.cu_frames)
        self.acc = to(data.acc_in)
        self.acc_in = self.acc.clone()
        self.n_frames = int(data.frame_type.shape[0])
        t_per = w.tokens_per_frame
        self.keep = torch.zeros((self.n_frames, t_per), dtype=torch.uint8, device=dev)
        self.kept_idx = torch.zeros((self.n_frames * t_per,), dtype=torch.int32, device=dev)
        self.kept_off = torch.zeros((self.n_frames + 1,), dtype=torch.int32, device=dev)
        self.ws_a_bytes = cs.cs_score_compact_workspace(w.n_streams, self.n_frames, w.grid_h, w.grid_w, w.group)
        self.ws_a = torch.zeros((max(8, self.ws_a_bytes),), dtype=torch.uint8, device=dev)
        # row lists
        n_reuse, n_q = int(data.info["n_reuse"]), int(data.info["n_q"])
        self.n_rows_true, self.n_q_true = n_reuse, n_q
        self.reuse_cap = n_reuse if reuse_cap is None else int(reuse_cap)
        self.q_cap = n_q if q_cap is None else int(q_cap)
        if self.q_cap < n_q or self.reuse_cap < n_reuse:
            raise ValueError("capacities below the step's row counts")
        if self.overlap is None and self.fused:
            # the fused launch wants the device to itself: its barrier waits for the whole grid to be resident
            self.overlap = False
        if self.overlap is None:
            # measured on MI355X: beside the layer loop the correction gains 1-4 % of the step once it
            # moves a gigabyte or more (32-64 streams, long dense windows) and loses 1-9 % below that,
            # where its calls are launch-bound
            elem = 2 if w.dtype == "bf16" else 4
            traffic = 4 * self.reuse_cap * w.n_layers * w.n_kv_heads * w.head_dim * elem
            self.overlap = traffic >= OVERLAP_MIN_BYTES
        self.side = torch.cuda.Stream() if self.overlap else None      # default priority
        old, new = data.old_layout, data.new_layout
        self.block_table = to(new.block_table)
        self.max_blocks = int(new.block_table.shape[1])
        if host_plan:
            p = data.plan
            pad = lambda a, n, fill: np.concatenate([a, np.full((n - a.shape[0],), fill, a.dtype)])
            self.src_slot, self.dst_slot = to(pad(p.src_slot, self.reuse_cap, -1)), to(pad(p.dst_slot, self.reuse_cap, -1))
            self.delta = to(pad(p.delta, self.reuse_cap, 0))
            self.q_slot, self.q_pos = to(pad(p.q_slot, self.q_cap, -1)), to(pad(p.q_pos, self.q_cap, 0))
            self.q_kind = to(pad(p.q_kind, self.q_cap, 0xFF))
            self.cu_q, self.kv_len = to(p.cu_q), to(p.kv_len)
        else:
            self.src_slot, self.dst_slot, self.delta = (i32(self.reuse_cap, -9) for _ in range(3))
            self.q_pos, self.q_slot = i32(self.q_cap, -9), i32(self.q_cap, -9)
            self.q_kind = torch.full((max(1, self.q_cap),), 7, dtype=torch.uint8, device=dev)
            self.cu_q, self.kv_len = i32(w.n_streams + 1, -9), i32(w.n_streams, -9)
        self.old_types, self.old_counts = to(old.frame_type), to(old.counts)
        self.bt_old = to(old.block_table)
        self.max_blocks_old = int(old.block_table.shape[1])
        self.new_types_out = torch.zeros_like(self.old_types)
        self.new_counts_out = torch.zeros_like(self.old_counts)
        self.totals = i32(4, -9)
        self.ws_p_bytes = cs.cs_plan_refresh_workspace(w.n_streams, w.window)
        self.ws_p = torch.zeros((max(8, self.ws_p_bytes),), dtype=torch.uint8, device=dev)
        # (b)
        self.k_pool = data.k_pool.to(dev)
        self.v_pool = data.v_pool.to(dev)
        self.stride_layer = self.k_pool.stride(0)
        self.stride_slot = self.k_pool.stride(1)
        self.stride_head = self.k_pool.stride(2)
        # (c), (d): rows beyond the step's own counts are padding (never read: slot -1 / beyond cu_q)
        grow = lambda t: t if self.q_cap == n_q else torch.cat(
            [t, torch.zeros((t.shape[0], self.q_cap - n_q) + tuple(t.shape[2:]), dtype=t.dtype, device=dev)], dim=1)
        self.q, self.k_new, self.v_new = grow(data.q.to(dev)), grow(data.k_new.to(dev)), grow(data.v_new.to(dev))
        self.out = torch.zeros_like(self.q)
        self.n_q = self.q_cap
        self.ws_d_bytes = cs.cs_window_prefill_attn_workspace(self.q_cap, w.n_streams, w.n_q_heads, w.n_kv_heads,
                                                              w.head_dim, self.max_blocks, self.dtype)
        self.ws_d = torch.zeros((max(8, self.ws_d_bytes),), dtype=torch.uint8, device=dev)

    def score_compact(self):
        w = self.data.workload
        self.cs.cs_score_compact(self.mv, self.sad, None, self.frame_type, self.cu_frames, self.acc,
                                 w.n_streams, self.n_frames, w.grid_h, w.grid_w, w.group, w.tau_mv_sq,
                                 w.tau_sad, w.use_residual, self.keep, self.kept_idx, self.kept_off,
                                 self.ws_a, self.ws_a_bytes)

    def scoring_status(self) -> int:
        """Status word of the last scoring call (synchronises): 0, or non-zero when a tile's bounded
        wait for its predecessor's count ran out and the compacted lists cannot be trusted."""
        import torch
        torch.cuda.synchronize()
        return self.cs.cs_score_compact_status(self.ws_a, self.ws_a_bytes)

    def plan_refresh(self):
        w = self.data.workload
        self.cs.cs_plan_refresh(self.old_types, self.old_counts, self.frame_type, self.kept_off, self.bt_old,
                                self.max_blocks_old, self.block_table, self.max_blocks, w.n_streams, w.window,
                                w.stride, w.n_text, w.tokens_per_frame, self.reuse_cap, self.q_cap,
                                self.src_slot, self.dst_slot, self.delta, self.q_pos, self.q_slot, self.q_kind,
                                self.cu_q, self.kv_len, self.new_types_out, self.new_counts_out, self.totals,
                                self.ws_p, self.ws_p_bytes)

    def rerotate(self, in_place: bool = False, layers=None):
        """Position correction of the reused rows; `layers` = (first, end) restricts the call to a range
        of layers (the rows of a layer are independent of every other layer's)."""
        w = self.data.workload
        if self.reuse_cap == 0:
            return
        l0, l1 = layers if layers is not None else (0, w.n_layers)
        self.cs.cs_kv_rerotate(self.k_pool[l0:l1], None if in_place else self.v_pool[l0:l1], self.src_slot,
                               None if in_place else self.dst_slot, self.delta,
                               int(self.src_slot.shape[0]) if self.reuse_cap else 0, l1 - l0, w.n_kv_heads,
                               w.head_dim, self.stride_layer, self.stride_slot, self.stride_head, w.rope_base,
                               self.cs.CS_ROPE_HALF_SPLIT, self.dtype)

    def refresh_scatter(self, layer: int):
        w = self.data.workload
        self.cs.cs_kv_refresh_scatter(self.k_new[layer], self.v_new[layer], self.q_slot,
                                      self.k_pool[layer], self.v_pool[layer], self.n_q, w.n_kv_heads,
                                      w.head_dim, self.stride_slot, self.stride_head, self.dtype)

    def attention(self, layer: int, reuse_plan: bool = False):
        """Attention of one layer.  The work plan depends only on cu_q / q_pos: `run` builds it at
        the first layer and lets the other layers reuse it."""
        w = self.data.workload
        self.cs.cs_window_prefill_attn(self.q[layer], self.k_pool[layer], self.v_pool[layer], self.cu_q,
                                       self.q_pos, self.kv_len, self.block_table, self.max_blocks,
                                       self.cs.CS_KV_BLOCK, self.out[layer], self.n_q, w.n_streams,
                                       w.n_q_heads, w.n_kv_heads, w.head_dim, self.stride_slot,
                                       self.stride_head, self.data.softmax_scale, self.dtype,
                                       self.ws_d if self.ws_d_bytes else None, self.ws_d_bytes,
                                       self.cs.CS_ATTN_PLAN_REUSE if reuse_plan else self.cs.CS_ATTN_PLAN_BUILD)

    def refresh_and_attention(self, layer: int, reuse_plan: bool = False):
        """Refresh write + attention of one layer as one call (one launch for bf16 / head_dim 128)."""
        w = self.data.workload
        self.cs.cs_refresh_prefill_attn(self.k_new[layer], self.v_new[layer], self.q_slot, self.n_q,
                                        self.q[layer], self.k_pool[layer], self.v_pool[layer], self.cu_q,
                                        self.q_pos, self.kv_len, self.block_table, self.max_blocks,
                                        self.cs.CS_KV_BLOCK, self.out[layer], self.n_q, w.n_streams,
                                        w.n_q_heads, w.n_kv_heads, w.head_dim, self.stride_slot,
                                        self.stride_head, self.data.softmax_scale, self.dtype,
                                        self.ws_d if self.ws_d_bytes else None, self.ws_d_bytes,
                                        self.cs.CS_ATTN_PLAN_REUSE if reuse_plan else self.cs.CS_ATTN_PLAN_BUILD)

    def attention_status(self) -> int:
        """Barrier status word of the fused launches (synchronises): 0 unless a launch's grid could not
        become resident as a whole."""
        import torch
        torch.cuda.synchronize()
        return self.cs.cs_attn_status(self.ws_d) if self.ws_d_bytes else 0

    def prepare(self):
        """Scoring and planning: everything the layer loop needs in device memory."""
        # scoring updates the accumulated mask in place; a repeated run (graph replay) starts from
        # the same mask so that every repetition plans the same step
        self.acc.copy_(self.acc_in)
        self.score_compact()
        if not self.host_plan:
            self.plan_refresh()

    def run(self):
        """One pass of the whole hot path."""
        import torch
        self.prepare()
        n_layers = self.data.workload.n_layers
        ready = {}
        if self.overlap and self.reuse_cap:
            # Sec. 3.5: the position correction needs the plan and the cached rows only, and layer l's
            # attention needs layer l's corrected rows only.  It is bandwidth work and attention is
            # matrix-core work, so it runs beside the layer loop on a second stream (fork and join
            # are stream waits, so a graph capture of this method records them as edges).
            main = torch.cuda.current_stream()
            self.side.wait_stream(main)
            with torch.cuda.stream(self.side):
                for l0 in range(0, n_layers, self.layers_per_rerotate):
                    l1 = min(n_layers, l0 + self.layers_per_rerotate)
                    self.rerotate(layers=(l0, l1))
                    ev = torch.cuda.Event()
                    ev.record(self.side)
                    ready[l0] = ev
        else:
            self.rerotate()
        for layer in range(n_layers):
            if layer in ready:
                # the refresh write touches other rows than the correction, but the fused call reads the cache too
                if self.fused:
                    torch.cuda.current_stream().wait_event(ready[layer])
            if self.fused:
                self.refresh_and_attention(layer, reuse_plan=layer > 0)
            else:
                self.refresh_scatter(layer)
                if layer in ready:
                    torch.cuda.current_stream().wait_event(ready[layer])
                self.attention(layer, reuse_plan=layer > 0)
        if ready:
            torch.cuda.current_stream().wait_stream(self.side)


DevicePlannedStep = DeviceStep     # former name of the device-planned step


@dataclass
class FrontEndData:
    """Inputs of a slide step that starts from decoder output: coding blocks, a motion field and
    the decoded luma planes of the S new frames of every stream (stream-major), the cached window,
    block tables sized for the largest window the step can produce, and capacity-sized Q/K/V."""
    workload: synth.Workload
    blocks: np.ndarray                 # synth.BLOCK_DTYPE records
    cu_blocks: np.ndarray              # int32 [F+1]
    field: np.ndarray                  # int16 [F, H/4, W/4, 2]
    cur: np.ndarray                    # uint8 [F, H, W]
    prev: np.ndarray
    frame_type: np.ndarray             # uint8 [F]
    cu_frames: np.ndarray              # int32 [B+1]
    acc_in: np.ndarray                 # uint8 [B, P]
    old_layout: planner.WindowLayout
    bt_new: np.ndarray                 # int32 [B, max_blocks]
    n_slots: int
    reuse_cap: int
    q_cap: int
    tau_res: int
    k_pool: object = None
    v_pool: object = None
    q: object = None
    k_new: object = None
    v_new: object = None
    softmax_scale: float = 0.0


def assemble_frontend_step(w: synth.Workload, scorer: Scorer, device="cpu", tau_res: Optional[int] = None) -> FrontEndData:
    """The cached window comes from scoring the history as in `assemble_step`; the S new frames
    arrive as decoder output.  How many of their tokens survive is only known on the device, so
    block tables, pool and the executed-row capacity allow for every token of a new frame."""
    meta = synth.batch_metadata(w)
    n_streams, hist, stride, window, t_per = w.n_streams, w.history, w.stride, w.window, w.tokens_per_frame
    past = hist - stride
    rows = meta.rows(0, past)
    cu = (np.arange(n_streams + 1) * past).astype(np.int32)
    _, _, off_h, acc_h = scorer(meta.mv[rows], meta.sad[rows], meta.frame_type[rows], cu,
                                np.zeros((n_streams, w.patches), np.uint8), w, w.tau_mv_sq, w.tau_sad)
    counts_h = np.diff(off_h).reshape(n_streams, past)
    old_counts = counts_h[:, past - window:].astype(np.int32)
    old_types = meta.frame_type.reshape(n_streams, hist)[:, past - window: past].astype(np.uint8)
    rows_new = meta.rows(past, stride)
    ftype = meta.frame_type[rows_new]
    blob = np.concatenate([synth.stream_metadata(w, s).blob[past:] for s in range(n_streams)])
    blocks, cu_blocks = synth.block_frames(w, ftype, blob)
    field = synth.motion_field(blocks, cu_blocks, 4)
    cur, prev = synth.decoded_frames(w, int(ftype.shape[0]), blob)

    overlap_types, overlap_counts = old_types[:, stride:], old_counts[:, stride:]
    old_len = old_counts.sum(axis=1) + w.n_text
    new_len_max = overlap_counts.sum(axis=1) + stride * t_per + w.n_text
    nb_old, nb_new = planner.blocks_needed(old_len), planner.blocks_needed(new_len_max)
    ids = synth.block_ids(w, int(nb_old.sum() + nb_new.sum()), tag=1)
    bt_old = np.zeros((n_streams, int(nb_old.max())), np.int32)
    bt_new = np.zeros((n_streams, int(nb_new.max())), np.int32)
    at = 0
    for s in range(n_streams):
        bt_old[s, : nb_old[s]] = ids[at: at + nb_old[s]]
        at += int(nb_old[s])
        bt_new[s, : nb_new[s]] = ids[at: at + nb_new[s]]
        at += int(nb_new[s])
    n_slots = int(ids.shape[0]) * synth.KV_BLOCK
    reused = int(overlap_counts[overlap_types != synth.FRAME_I].sum())
    anchors = int(overlap_counts[overlap_types == synth.FRAME_I].sum())
    q_cap = anchors + n_streams * (stride * t_per + w.n_text)
    data = FrontEndData(w, blocks, cu_blocks, field, cur, prev, ftype, (np.arange(n_streams + 1) * stride).astype(np.int32),
                        acc_h, planner.WindowLayout(old_types, old_counts, w.n_text, bt_old), bt_new, n_slots,
                        reused, q_cap, int(0.05 * 255 * 256) if tau_res is None else int(tau_res),
                        softmax_scale=1.0 / math.sqrt(w.head_dim))
    shape_pool = (w.n_layers, n_slots, w.n_kv_heads, w.head_dim)
    data.k_pool = synth.normal_tensor(w, (11,), shape_pool, device)
    data.v_pool = synth.normal_tensor(w, (12,), shape_pool, device)
    data.q = synth.normal_tensor(w, (13,), (w.n_layers, q_cap, w.n_q_heads, w.head_dim), device)
    data.k_new = synth.normal_tensor(w, (14,), (w.n_layers, q_cap, w.n_kv_heads, w.head_dim), device)
    data.v_new = synth.normal_tensor(w, (15,), (w.n_layers, q_cap, w.n_kv_heads, w.head_dim), device)
    return data


class FrontEndStep:
    """The whole chain on the GPU, queued without a host round trip: block projection and residual
    proxy (decoder output -> per-patch metadata), scoring + compaction, refresh plan, position
    correction of the reused rows, then per layer refresh write and attention."""

    def __init__(self, data: FrontEndData):
        import torch
        from . import binding as cs
        self.cs, self.data = cs, data
        w = data.workload
        dev = self.dev = torch.device("cuda")
        to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        self.dtype = cs.CS_BF16 if w.dtype == "bf16" else cs.CS_F32
        self.n_frames = int(data.frame_type.shape[0])
        self.src_w, self.src_h = synth.SOURCE_SIZE
        self.in_w, self.in_h = synth.input_size(w)
        self.blocks = to(data.blocks.view(np.uint8))
        self.n_blocks = int(data.blocks.shape[0])
        self.cu_blocks, self.field, self.cur, self.prev = to(data.cu_blocks), to(data.field), to(data.cur), to(data.prev)
        self.frame_type, self.cu_frames = to(data.frame_type), to(data.cu_frames)
        self.acc, self.acc_in = to(data.acc_in), to(data.acc_in)
        i32 = lambda shape, fill=0: torch.full(shape, fill, dtype=torch.int32, device=dev)
        self.mv = torch.zeros((self.n_frames, w.patches, 2), dtype=torch.int16, device=dev)
        self.intra = torch.zeros((self.n_frames, w.patches), dtype=torch.uint8, device=dev)
        self.res = i32((self.n_frames, w.patches))
        t_per = w.tokens_per_frame
        self.keep = torch.zeros((self.n_frames, t_per), dtype=torch.uint8, device=dev)
        self.kept_idx, self.kept_off = i32((self.n_frames * t_per,)), i32((self.n_frames + 1,))
        self.ws_a_bytes = cs.cs_score_compact_workspace(w.n_streams, self.n_frames, w.grid_h, w.grid_w, w.group)
        self.ws_a = torch.zeros((max(8, self.ws_a_bytes),), dtype=torch.uint8, device=dev)
        old = data.old_layout
        self.old_types, self.old_counts = to(old.frame_type), to(old.counts)
        self.bt_old, self.bt_new = to(old.block_table), to(data.bt_new)
        self.max_blocks_old, self.max_blocks = int(old.block_table.shape[1]), int(data.bt_new.shape[1])
        self.reuse_cap, self.q_cap = data.reuse_cap, data.q_cap
        self.src_slot, self.dst_slot, self.delta = (i32((max(1, self.reuse_cap),), -9) for _ in range(3))
        self.q_pos, self.q_slot = i32((self.q_cap,), -9), i32((self.q_cap,), -9)
        self.q_kind = torch.full((self.q_cap,), 7, dtype=torch.uint8, device=dev)
        self.cu_q, self.kv_len, self.totals = i32((w.n_streams + 1,)), i32((w.n_streams,)), i32((4,))
        self.new_types, self.new_counts = torch.zeros_like(self.old_types), torch.zeros_like(self.old_counts)
        self.ws_p_bytes = cs.cs_plan_refresh_workspace(w.n_streams, w.window)
        self.ws_p = torch.zeros((max(8, self.ws_p_bytes),), dtype=torch.uint8, device=dev)
        self.k_pool, self.v_pool = data.k_pool.to(dev), data.v_pool.to(dev)
        self.stride_layer, self.stride_slot, self.stride_head = (self.k_pool.stride(i) for i in range(3))
        self.q, self.k_new, self.v_new = data.q.to(dev), data.k_new.to(dev), data.v_new.to(dev)
        self.out = torch.zeros_like(self.q)
        self.ws_d_bytes = cs.cs_window_prefill_attn_workspace(self.q_cap, w.n_streams, w.n_q_heads, w.n_kv_heads,
                                                              w.head_dim, self.max_blocks, self.dtype)
        self.ws_d = torch.zeros((max(8, self.ws_d_bytes),), dtype=torch.uint8, device=dev)

    def front_end(self):
        w, cs = self.data.workload, self.cs
        cs.cs_project_blocks(self.blocks, self.cu_blocks, self.n_frames, self.src_w, self.src_h, self.in_w, self.in_h,
                             synth.MODEL_PATCH, w.grid_h, w.grid_w, self.mv, self.intra, n_blocks=self.n_blocks)
        cs.cs_residual_proxy(self.cur, self.prev, self.field, self.n_frames, self.src_w, self.src_h, self.src_w,
                             self.src_w * self.src_h, 4, self.in_w, self.in_h, synth.MODEL_PATCH, w.grid_h, w.grid_w,
                             self.res)

    def score_and_plan(self):
        w, cs = self.data.workload, self.cs
        self.acc.copy_(self.acc_in)                       # a repeated run plans the same step
        cs.cs_score_compact(self.mv, self.res, self.intra, self.frame_type, self.cu_frames, self.acc, w.n_streams,
                            self.n_frames, w.grid_h, w.grid_w, w.group, w.tau_mv_sq, self.data.tau_res, True, self.keep,
                            self.kept_idx, self.kept_off, self.ws_a, self.ws_a_bytes)
        cs.cs_plan_refresh(self.old_types, self.old_counts, self.frame_type, self.kept_off, self.bt_old,
                           self.max_blocks_old, self.bt_new, self.max_blocks, w.n_streams, w.window, w.stride, w.n_text,
                           w.tokens_per_frame, self.reuse_cap, self.q_cap, self.src_slot, self.dst_slot, self.delta,
                           self.q_pos, self.q_slot, self.q_kind, self.cu_q, self.kv_len, self.new_types, self.new_counts,
                           self.totals, self.ws_p, self.ws_p_bytes)

    def kv_and_attention(self):
        w, cs = self.data.workload, self.cs
        if self.reuse_cap > 0:
            cs.cs_kv_rerotate(self.k_pool, self.v_pool, self.src_slot, self.dst_slot, self.delta, self.reuse_cap,
                              w.n_layers, w.n_kv_heads, w.head_dim, self.stride_layer, self.stride_slot, self.stride_head,
                              w.rope_base, cs.CS_ROPE_HALF_SPLIT, self.dtype)
        for layer in range(w.n_layers):
            cs.cs_kv_refresh_scatter(self.k_new[layer], self.v_new[layer], self.q_slot, self.k_pool[layer],
                                     self.v_pool[layer], self.q_cap, w.n_kv_heads, w.head_dim, self.stride_slot,
                                     self.stride_head, self.dtype)
            cs.cs_window_prefill_attn(self.q[layer], self.k_pool[layer], self.v_pool[layer], self.cu_q, self.q_pos,
                                      self.kv_len, self.bt_new, self.max_blocks, cs.CS_KV_BLOCK, self.out[layer],
                                      self.q_cap, w.n_streams, w.n_q_heads, w.n_kv_heads, w.head_dim, self.stride_slot,
                                      self.stride_head, self.data.softmax_scale, self.dtype,
                                      self.ws_d if self.ws_d_bytes else None, self.ws_d_bytes,
                                      cs.CS_ATTN_PLAN_REUSE if layer > 0 else cs.CS_ATTN_PLAN_BUILD)

    def run(self):
        self.front_end()
        self.score_and_plan()
        self.kv_and_attention()
