#!/usr/bin/env python3
"""Benchmark of the codec-guided window-prefill step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic streams:
  cs_score_compact -> cs_kv_rerotate (all layers) -> per layer: cs_kv_refresh_scatter,
  cs_window_prefill_attn.
Inputs are resident in HBM before the timed region starts.  The step is captured once in a HIP
graph and the timed region replays it K times (the refresh plan is built beforehand from an
identical, untimed run of the scoring kernel; planning on the host is not part of the timed step).

Printed: ONE JSON line with the whole-job throughput (executed tokens per second), a `roofline`
object for the dominant kernel (event-timed on the launch stream) and a `cpu_baseline` object (the
CPU oracle timed on this machine's host cores on a bounded sample of the same workload).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_MFMA_BF16_TFLOPS = 2500.0  # dense bf16
DEFAULT_WORKLOAD = "cfg1_qwen7b_1stream"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD,
                    help="one of the synthetic workloads in paper_2604_06036_amd.synth.WORKLOADS")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--eager", action="store_true", help="launch from Python instead of replaying a HIP graph")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference for HBM counters and copy bandwidth)")
    ap.add_argument("--no-frontend-step", action="store_true",
                    help="skip the leg that runs the chain from decoder output to attention output")
    ap.add_argument("--no-device-plan", action="store_true",
                    help="skip the leg that runs the step with the refresh plan made on the GPU")
    ap.add_argument("--no-scaled-scoring", action="store_true",
                    help="skip the scaled-batch bandwidth measurement of cs_score_compact")
    return ap.parse_args()


def kernel_bytes_flops(w, info, n_layers):
    """Algorithmic work per launch of each kernel (what the method itself must move / compute)."""
    e = 2 if w.dtype == "bf16" else 4
    row = w.n_kv_heads * w.head_dim * e
    n_frames = w.n_streams * w.stride
    patches = n_frames * w.patches
    tokens = n_frames * w.tokens_per_frame
    a_bytes = patches * (4 + (4 if w.use_residual else 0) + 2) + tokens * 1 + info["kept_new"] * 4 + (n_frames + 1) * 4
    b_bytes = info["n_reuse"] * (n_layers * 4 * row + 12)          # K read+write, V read+write, 3 index words
    c_bytes = info["n_q"] * (4 * row + 4)                           # K,V new read + K,V cache write + slot
    d_flops = 4.0 * w.head_dim * w.n_q_heads * info["visible_pairs"]
    d_bytes = 2 * info["kv_len_total"] * row + 2 * info["n_q"] * w.n_q_heads * w.head_dim * e
    return dict(a_bytes=a_bytes, b_bytes=b_bytes, c_bytes=c_bytes, d_flops=d_flops, d_bytes=d_bytes)


def event_time(torch, fn, reps):
    """Average milliseconds of fn(), bracketed by HIP events on the current (launch) stream."""
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) / reps


def copy_calibration(torch):
    """A plain device-to-device copy of known size: 1 GiB read + 1 GiB written (larger than the
    256 MB Infinity Cache).  Its HBM counters calibrate FETCH_SIZE / WRITE_SIZE, its rate is the
    practical ceiling the bandwidth-bound kernels are compared with."""
    n = 1 << 29                                             # bf16 elements = 1 GiB
    a = torch.ones((n,), dtype=torch.bfloat16, device="cuda")
    b = torch.empty_like(a)
    for _ in range(2):
        b.copy_(a)
    ms = event_time(torch, lambda: b.copy_(a), 5)
    return dict(bytes_read=2 * n, bytes_written=2 * n, ms=ms, GBps=4.0 * n / ms / 1e6)


def scaled_scoring(w, torch, binding):
    """cs_score_compact on a SCALED batch: the workload's per-stream shape (one new frame of the
    same patch grid per stream) with the stream count raised until the metadata exceeds 256 MB, so
    that the kernel's bandwidth rather than its launch latency is measured.  Metadata is drawn on
    the GPU with the generator's marginals (25 % of patches moving), without the blob structure."""
    n_patch = w.patches
    n_streams = max(w.n_streams, (288 << 20) // (n_patch * 8))
    gen = torch.Generator(device="cuda")
    gen.manual_seed(0xC0DEC)
    moving = torch.rand((n_streams, n_patch), generator=gen, device="cuda") < 0.25
    sigma = torch.where(moving, 24.0, 1.0).unsqueeze(-1)
    mv = torch.round(torch.randn((n_streams, n_patch, 2), generator=gen, device="cuda") * sigma).to(torch.int16)
    sad = torch.round(torch.empty((n_streams, n_patch), device="cuda").exponential_(1 / 100.0, generator=gen)
                      * torch.where(moving, 10.0, 1.0)).to(torch.int32)
    ftype = (torch.rand((n_streams,), generator=gen, device="cuda") < 0.125).to(torch.uint8)
    cu = torch.arange(n_streams + 1, dtype=torch.int32, device="cuda")
    acc = (torch.rand((n_streams, n_patch), generator=gen, device="cuda") < 0.05).to(torch.uint8)
    t_per = w.tokens_per_frame
    keep = torch.empty((n_streams, t_per), dtype=torch.uint8, device="cuda")
    idx = torch.empty((n_streams * t_per,), dtype=torch.int32, device="cuda")
    off = torch.empty((n_streams + 1,), dtype=torch.int32, device="cuda")
    wsb = binding.cs_score_compact_workspace(n_streams, n_streams, w.grid_h, w.grid_w, w.group)
    ws = torch.empty((wsb,), dtype=torch.uint8, device="cuda")
    del moving, sigma
    call = lambda: binding.cs_score_compact(mv, sad, None, ftype, cu, acc, n_streams, n_streams, w.grid_h,
                                            w.grid_w, w.group, w.tau_mv_sq, w.tau_sad, True, keep, idx, off,
                                            ws, wsb)
    for _ in range(2):
        call()
    ms = event_time(torch, call, 5)
    kept = int(off[-1].item())
    p_frames = int((ftype == 0).sum().item())
    # P-frames read MV + SAD + acc and write keep (acc writes only where it changes: not counted);
    # I-frames write keep + acc; every kept token writes a 4-byte id; one offset per frame
    nbytes = p_frames * n_patch * (4 + 4 + 1 + 1) + (n_streams - p_frames) * n_patch * 2 + kept * 4 + n_streams * 4
    return dict(label="scaled batch", streams=n_streams, patches=n_streams * n_patch, kept=kept, ms=ms,
                bytes=nbytes, GBps=nbytes / ms / 1e6, frac_of_hbm_peak=nbytes / ms / 1e6 / PEAK_HBM_GBS)


def block_projection(w, torch, binding, reps):
    """cs_project_blocks: decoder-shaped block lists (macroblock partitions of a 1920 x 1080 frame)
    to the workload's patch grid.  Real shape = the step's own new frames; scaled = the same frames
    repeated until the block records exceed 256 MB (bandwidth rather than launch latency)."""
    import numpy as np
    from paper_2604_06036_amd import synth
    src_w, src_h = synth.SOURCE_SIZE
    in_w, in_h = synth.input_size(w)
    ftypes, blobs = [], []
    for s in range(min(w.n_streams, 64)):
        m = synth.stream_metadata(w, s)
        ftypes.append(m.frame_type[-w.stride:])
        blobs.append(m.blob[-w.stride:])
    blocks, cu = synth.block_frames(w, np.concatenate(ftypes), np.concatenate(blobs))
    out = {}
    for label in ("real shape", "scaled batch"):
        n_frames, n_blocks = int(cu.shape[0]) - 1, int(blocks.shape[0])
        d_blocks = torch.from_numpy(blocks.view(np.uint8).copy()).cuda()
        d_cu = torch.from_numpy(cu).cuda()
        mv = torch.empty((n_frames, w.patches, 2), dtype=torch.int16, device="cuda")
        intra = torch.empty((n_frames, w.patches), dtype=torch.uint8, device="cuda")
        call = lambda: binding.cs_project_blocks(d_blocks, d_cu, n_frames, src_w, src_h, in_w, in_h,
                                                 synth.MODEL_PATCH, w.grid_h, w.grid_w, mv, intra, n_blocks=n_blocks)
        for _ in range(2):
            call()
        ms = event_time(torch, call, reps)
        nbytes = n_blocks * 16 + n_frames * (w.patches * 5 + 4)
        out[label] = dict(frames=n_frames, blocks=n_blocks, ms=ms, bytes=nbytes, GBps=nbytes / ms / 1e6,
                          frac_of_hbm_peak=nbytes / ms / 1e6 / PEAK_HBM_GBS)
        if label == "real shape":
            rep = max(1, (288 << 20) // max(1, n_blocks * 16))
            off = (np.arange(rep, dtype=np.int64)[:, None] * n_blocks + cu[None, :-1]).reshape(-1)
            cu = np.concatenate([off, [rep * n_blocks]]).astype(np.int32)
            blocks = np.tile(blocks, rep)
        del d_blocks, mv, intra
    return out


def residual_proxy(w, torch, binding, reps):
    """cs_residual_proxy on 1920 x 1080 luma planes with a 4 x 4-pixel motion field: real shape = one
    new frame per stream (at most 32 streams drawn), scaled = the same planes repeated until current
    + previous frames exceed 256 MB."""
    import numpy as np
    from paper_2604_06036_amd import synth
    src_w, src_h = synth.SOURCE_SIZE
    in_w, in_h = synth.input_size(w)
    n_real = min(w.n_streams * w.stride, 32)
    metas = [synth.stream_metadata(w, s) for s in range(min(w.n_streams, n_real))]
    ftype = np.concatenate([m.frame_type[-w.stride:] for m in metas])[:n_real]
    blob = np.concatenate([m.blob[-w.stride:] for m in metas])[:n_real]
    blocks, cu = synth.block_frames(w, ftype, blob)
    field = torch.from_numpy(synth.motion_field(blocks, cu, 4)).cuda()
    cur, prev = (torch.from_numpy(a).cuda() for a in synth.decoded_frames(w, n_real, blob))
    out = {}
    for label in ("real shape", "scaled batch"):
        n_frames = int(cur.shape[0])
        res = torch.empty((n_frames, w.patches), dtype=torch.int32, device="cuda")
        call = lambda: binding.cs_residual_proxy(cur, prev, field, n_frames, src_w, src_h, src_w, src_w * src_h, 4,
                                                 in_w, in_h, synth.MODEL_PATCH, w.grid_h, w.grid_w, res)
        for _ in range(2):
            call()
        ms = event_time(torch, call, reps)
        nbytes = n_frames * (2 * src_w * src_h + field.shape[1] * field.shape[2] * 4 + w.patches * 4)
        out[label] = dict(frames=n_frames, ms=ms, bytes=nbytes, GBps=nbytes / ms / 1e6,
                          frac_of_hbm_peak=nbytes / ms / 1e6 / PEAK_HBM_GBS)
        if label == "real shape":
            rep = max(1, -(-(160 << 20) // (n_frames * src_w * src_h)))
            cur, prev, field = cur.repeat(rep, 1, 1), prev.repeat(rep, 1, 1), field.repeat(rep, 1, 1, 1)
    return out


def axes_rerotation(w, step, torch, binding, b_bytes, reps):
    """cs_kv_rerotate_axes (three-axis RoPE correction) on the step's own reuse plan: the window
    slides in time only, so the shift is (delta, 0, 0); frequency pairs are mapped to (t, h, w) in
    sections of 1/4, 3/8, 3/8 of the pairs (the 16/24/24 split of a 128-wide head).  Same bytes
    as the one-dimensional call."""
    half = w.head_dim // 2
    n_t = half // 4
    n_h = (half - n_t) // 2
    axis = torch.cat([torch.zeros(n_t), torch.ones(n_h), torch.full((half - n_t - n_h,), 2.0)]).to(torch.uint8).cuda()
    delta3 = torch.stack([step.delta, torch.zeros_like(step.delta), torch.zeros_like(step.delta)], dim=1).contiguous()
    call = lambda: binding.cs_kv_rerotate_axes(
        step.k_pool, step.v_pool, step.src_slot, step.dst_slot, delta3, axis, int(step.src_slot.shape[0]),
        w.n_layers, w.n_kv_heads, w.head_dim, step.stride_layer, step.stride_slot, step.stride_head, w.rope_base,
        binding.CS_ROPE_HALF_SPLIT, step.dtype)
    call()
    ms = event_time(torch, call, reps)
    return dict(ms=ms, bytes=b_bytes, GBps=b_bytes / ms / 1e6, frac_of_hbm_peak=b_bytes / ms / 1e6 / PEAK_HBM_GBS,
                sections=[n_t, n_h, half - n_t - n_h])


def device_planned(w, data, torch, engine, steps, warmup):
    """The same step with the refresh plan made on the GPU between scoring and re-rotation
    (cs_plan_refresh), captured in a HIP graph: nothing passes through the host inside the step.
    Row lists are sized to capacities 1/8 above the step's row counts, rounded up to 256; the
    consumers run over the capacities and skip the padding.  For comparison, the host route the
    default step keeps outside its timed region: copy the offsets back, plan on the host, copy the
    lists to the device."""
    import numpy as np
    from paper_2604_06036_amd import planner
    cap = lambda n: (n + n // 8 + 255) // 256 * 256
    info = data.info
    step = engine.DevicePlannedStep(data, reuse_cap=cap(info["n_reuse"]), q_cap=cap(info["n_q"]))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step.run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    totals = step.totals.cpu().tolist()
    if totals != [info["n_reuse"], info["n_q"], 0, 0]:
        raise RuntimeError(f"device plan totals {totals} differ from the host plan's")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step.run()
    for _ in range(warmup):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    ms_step = 1e3 * (time.perf_counter() - t0) / steps
    t_plan = event_time(torch, step.plan_refresh, max(3, min(steps, 20)))

    def host_route():
        off = step.kept_off.cpu().numpy()                                   # waits for the scoring call
        counts = np.diff(off).reshape(w.n_streams, w.stride).astype(np.int32)
        types = data.frame_type.reshape(w.n_streams, w.stride)
        pl = planner.plan_slide(data.old_layout, types, counts, data.plan.layout.block_table, w.tokens_per_frame)
        for a in (pl.src_slot, pl.dst_slot, pl.delta, pl.q_pos, pl.q_slot, pl.cu_q, pl.kv_len):
            torch.from_numpy(a).to("cuda")
        torch.cuda.synchronize()
    host_route()
    t0 = time.perf_counter()
    for _ in range(5):
        host_route()
    ms_host = 1e3 * (time.perf_counter() - t0) / 5
    return dict(ms_per_step=ms_step, tokens_per_s=info["n_q"] / (ms_step * 1e-3), plan_call_ms=t_plan,
                reuse_cap=step.reuse_cap, q_cap=step.q_cap, host_route_ms=ms_host)


def frontend_step(w, torch, engine, steps, warmup):
    """The chain from decoder output to attention output in one HIP graph: block projection,
    residual proxy, scoring with rescue, refresh plan on the GPU, position correction, then per
    layer refresh write + attention, on lists sized to the step's capacities (every token of a new
    frame may be kept).  Its executed-token count comes from the device plan."""
    data = engine.assemble_frontend_step(w, engine.hip_scorer, device="cuda")
    step = engine.FrontEndStep(data)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step.run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    totals = step.totals.cpu().tolist()
    if totals[2] != 0:
        raise RuntimeError(f"front-end step: plan flags {totals}")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step.run()
    for _ in range(warmup):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    ms = 1e3 * (time.perf_counter() - t0) / steps
    t_front = event_time(torch, step.front_end, max(3, min(steps, 20)))
    t_plan = event_time(torch, step.score_and_plan, max(3, min(steps, 20)))
    return dict(ms_per_step=ms, executed_tokens=totals[1], reused_rows=totals[0], q_cap=data.q_cap,
                tokens_per_s=totals[1] / (ms * 1e-3), front_end_ms=t_front, score_and_plan_ms=t_plan,
                frames=int(data.frame_type.shape[0]), blocks=int(data.blocks.shape[0]))


def cpu_baseline(w, data, step, torch):
    """The oracle, as it stands, on the host: scoring, re-rotation of every reused row for all
    layers, then refresh write + attention for a bounded number of layers, scaled to all layers."""
    import numpy as np
    from oracle import codecsight_oracle as oc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    p = data.plan
    f64 = lambda t: t.detach().cpu().float().numpy().astype(np.float64)
    pairs_per_layer = w.n_q_heads * data.info["visible_pairs"]
    # keep the sample near 10-30 s: the fp64 oracle sustains very roughly 2e9 pair-dims/s per core
    budget_pairs = 1.0e9 * max(1, cores)
    n_l = int(max(1, min(w.n_layers, budget_pairs // max(1.0, pairs_per_layer * w.head_dim / 64))))
    max_rows = 4096
    rows = p.src_slot.shape[0]
    pick = np.arange(rows) if rows <= max_rows else np.sort(np.random.default_rng(0).choice(rows, max_rows, replace=False))
    k_host = step.k_pool_before[:, torch.from_numpy(p.src_slot[pick].astype(np.int64)).to(step.dev)].cpu()
    t0 = time.perf_counter()
    oc.score_compact(data.mv, data.sad if w.use_residual else None, None, data.frame_type, data.cu_frames,
                     data.acc_in, w.grid_h, w.grid_w, w.group, w.tau_mv_sq, w.tau_sad, w.use_residual)
    t_a = time.perf_counter() - t0
    t0 = time.perf_counter()
    oc.rotate(f64(k_host), p.delta[pick].astype(np.float64)[None, :, None], w.rope_base)
    t_b = (time.perf_counter() - t0) * rows / max(1, pick.size)
    # layers: cache after (b) is taken as given (copying device results to the host is not timed)
    q_sel = None
    n_q = int(p.q_pos.size)
    max_q = 2048
    qrows = None if n_q <= max_q else np.sort(np.random.default_rng(1).choice(n_q, max_q, replace=False))
    t_cd = 0.0
    for layer in range(n_l):
        k_l, v_l = f64(step.k_pool[layer]), f64(step.v_pool[layer])
        kn, vn, q_l = f64(step.k_new[layer]), f64(step.v_new[layer]), f64(step.q[layer])
        t0 = time.perf_counter()
        oc.scatter(k_l, kn, p.q_slot)
        oc.scatter(v_l, vn, p.q_slot)
        t_c = time.perf_counter() - t0
        t0 = time.perf_counter()
        oc.window_attn(q_l, k_l, v_l, p.cu_q, p.q_pos, p.layout.block_table, w.n_q_heads,
                       data.softmax_scale, rows=qrows)
        t_d = (time.perf_counter() - t0) * (1.0 if qrows is None else n_q / qrows.size)
        t_cd += t_c + t_d
    t_step = t_a + t_b + w.n_layers * t_cd / n_l
    sample = (f"oracle: scoring of the step's frames; re-rotation of {pick.size} of {rows} reused rows x "
              f"{w.n_layers} layers (scaled to all rows); refresh write + attention of {n_l} of {w.n_layers} "
              f"layers" + ("" if qrows is None else f" on {qrows.size} of {n_q} queries") + " (scaled to the full step)")
    return dict(value=n_q / t_step, unit="tokens/s", cores=int(cores), kind="oracle", sample=sample,
                seconds_per_step=t_step)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the path shards by stream with no exchange step; "
              "no multi-GPU figure is produced). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2604_06036_amd import binding, engine, synth

    if not os.path.exists(binding.LIB_PATH):
        print("bench.py: libcodecsight.so is missing; run `python -m paper_2604_06036_amd.build` "
              "(there is no CPU fallback)", file=sys.stderr)
        sys.exit(3)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    w = synth.WORKLOADS[args.workload]
    t_setup = time.perf_counter()
    data = engine.assemble_step(w, engine.hip_scorer, device="cuda")
    step = engine.DeviceStep(data)
    step.k_pool_before = step.k_pool.clone()     # pre-step cache, for the CPU baseline's re-rotation leg
    info = data.info
    work = kernel_bytes_flops(w, info, w.n_layers)
    print(f"[bench] {w.name}: {info} setup {time.perf_counter() - t_setup:.1f}s", file=sys.stderr, flush=True)

    # ---- the timed region: W warm-up steps, then exactly K steps
    launch = "eager"
    run_step = step.run
    graph = None
    if not args.eager:
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                step.run()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                step.run()
            run_step = graph.replay
            launch = "hipgraph"
        except Exception as exc:  # capture unsupported: fall back to eager launches, and say so
            print(f"[bench] graph capture failed ({exc}); using eager launches", file=sys.stderr)
            run_step, launch = step.run, "eager"
    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    tokens_per_s = info["n_q"] / (ms_per_step * 1e-3)

    # ---- per-kernel clocks: HIP events on the launch stream around back-to-back launches
    L = w.n_layers
    reps = max(3, min(args.steps, 20))
    t_a = event_time(torch, step.score_compact, reps)
    t_b = event_time(torch, step.rerotate, reps)
    t_c = event_time(torch, lambda: [step.refresh_scatter(l) for l in range(L)], reps) / L
    t_d = event_time(torch, lambda: [step.attention(l, reuse_plan=l > 0) for l in range(L)], reps) / L
    kernels = {
        "cs_score_compact": dict(ms=t_a, launches_per_step=1, GBps=work["a_bytes"] / t_a / 1e6),
        "cs_kv_rerotate": dict(ms=t_b, launches_per_step=1, GBps=work["b_bytes"] / t_b / 1e6),
        "cs_kv_refresh_scatter": dict(ms=t_c, launches_per_step=L, GBps=work["c_bytes"] / t_c / 1e6),
        "cs_window_prefill_attn": dict(ms=t_d, launches_per_step=L, TFLOPs=work["d_flops"] / t_d / 1e9,
                                       GBps=work["d_bytes"] / t_d / 1e6),
    }
    share = {k: v["ms"] * v["launches_per_step"] for k, v in kernels.items()}
    dominant = max(share, key=share.get)
    # HBM bytes per launch of the dominant kernel, from committed rocprofv3 --pmc FETCH_SIZE /
    # WRITE_SIZE runs of this same command, calibrated against a 1 GiB copy (profiles/): not
    # measured live, null when no such run exists for this workload
    traffic, traffic_detail = None, None
    tpath = os.path.join(ROOT, "profiles", "pmc_traffic.json")
    if os.path.exists(tpath):
        try:
            per_wl = json.load(open(tpath)).get(w.name, {})
            traffic_detail = per_wl.get(dominant)
            if traffic_detail:
                traffic = traffic_detail["read_bytes"] + traffic_detail["write_bytes"]
                merge = per_wl.get("attn_merge") if dominant == "cs_window_prefill_attn" else None
                if merge:                                    # split sweeps: the call is two kernels
                    traffic += merge["read_bytes"] + merge["write_bytes"]
                    traffic_detail = dict(traffic_detail, merge_kernel=merge)
        except Exception:
            traffic, traffic_detail = None, None
    if dominant == "cs_window_prefill_attn":
        ach = kernels[dominant]["TFLOPs"]
        roofline = dict(bound="mfma", kernel=("window_attn_bf16_stream_kernel (+ window_attn_merge_kernel where the key sweep is split)"
                                if w.dtype == "bf16" and w.head_dim == 128 else
                                "window_attn_bf16_kernel" if w.dtype == "bf16" else "window_attn_f32_kernel"),
                        achieved=ach, peak=PEAK_MFMA_BF16_TFLOPS, unit="TFLOP/s", frac=ach / PEAK_MFMA_BF16_TFLOPS,
                        traffic=traffic, traffic_detail=traffic_detail, algorithmic_bytes=work["d_bytes"],
                        flops_per_launch=work["d_flops"], ms_per_launch=t_d)
    else:
        ach = kernels[dominant]["GBps"]
        key = {"cs_score_compact": "a_bytes", "cs_kv_rerotate": "b_bytes", "cs_kv_refresh_scatter": "c_bytes"}[dominant]
        roofline = dict(bound="hbm", kernel=dominant, achieved=ach, peak=PEAK_HBM_GBS, unit="GB/s",
                        frac=ach / PEAK_HBM_GBS, traffic=traffic, traffic_detail=traffic_detail, bytes_per_launch=work[key],
                        ms_per_launch=kernels[dominant]["ms"])

    out = {
        "metric": "window-prefill tokens/s per MI355X (executed refresh+new+text tokens per second, whole step)",
        "value": tokens_per_s,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "streams": w.n_streams, "layers": w.n_layers,
                   "heads": f"{w.n_q_heads}/{w.n_kv_heads}", "head_dim": w.head_dim,
                   "window_frames": w.window, "stride_frames": w.stride, "tokens_per_frame": w.tokens_per_frame,
                   "executed_tokens": info["n_q"], "reused_rows": info["n_reuse"],
                   "window_tokens": info["kv_len_total"], "launch": launch},
        "window_tokens_per_s": info["kv_len_total"] / (ms_per_step * 1e-3),
        "kernels": kernels,
        "roofline": roofline,
    }
    if args.calibrate_copy:
        out["copy_calibration"] = copy_calibration(torch)
    if not args.no_scaled_scoring:
        out["score_compact_scaled"] = scaled_scoring(w, torch, binding)
        out["block_projection"] = block_projection(w, torch, binding, reps)
        out["residual_proxy"] = residual_proxy(w, torch, binding, reps)
        out["kv_rerotate_axes"] = axes_rerotation(w, step, torch, binding, work["b_bytes"], reps)
    if not args.no_frontend_step:
        out["frontend_step"] = frontend_step(w, torch, engine, args.steps, args.warmup)
    if not args.no_device_plan:
        out["device_planned_step"] = device_planned(w, data, torch, engine, args.steps, args.warmup)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, data, step, torch)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
