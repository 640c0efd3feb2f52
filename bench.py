#!/usr/bin/env python3
"""Benchmark of the codec-guided window-prefill step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic streams, with nothing
passing through the host in between:
  cs_score_compact -> cs_plan_refresh -> cs_kv_rerotate (all layers) -> per layer:
  cs_kv_refresh_scatter, cs_window_prefill_attn.
Inputs are resident in HBM before the timed region starts.  The step is captured once in a HIP
graph and the timed region replays it K times.

By default all five bf16 workloads are measured one after the other (the one-stream shape, the
32-stream batch, both readings of the long window, the 64-stream batch); the top-level `value`,
`ms_per_step`, `config` and `roofline` are those of the LAST one, the largest (64 streams, 32
layers), and `workloads` carries the same figures for each.  `--workload NAME` measures one.

Printed: ONE JSON line with the whole-job throughput (executed tokens per second), a `roofline`
object for the dominant kernel (event-timed on the launch stream), per-kernel rooflines, and a
`cpu_baseline` object (the CPU oracle timed on this machine's host cores on a bounded sample of the
headline workload, on all cores and on one).
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
DEFAULT_WORKLOADS = ("cfg1_qwen7b_1stream", "cfg2_qwen7b_32streams", "cfg3p_longwindow_pruned",
                     "cfg3d_longwindow_dense", "cfg4_internlm7b_64streams")   # the last one is the headline


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=None,
                    help="measure this workload only (a name in paper_2604_06036_amd.synth.WORKLOADS); "
                         "default: all five bf16 workloads, the 64-stream batch as the headline")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--eager", action="store_true", help="launch from Python instead of replaying a HIP graph")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference for HBM counters and copy bandwidth)")
    ap.add_argument("--no-overlap", action="store_true",
                    help="queue the position correction as one call ahead of the layer loop on every workload "
                         "(the schedule the per-call counters in profiles/ are taken with)")
    ap.add_argument("--no-fused-step", action="store_true",
                    help="skip the leg that times the step with refresh write and attention in one launch")
    ap.add_argument("--no-frontend-step", action="store_true",
                    help="skip the leg that runs the chain from decoder output to attention output")
    ap.add_argument("--no-host-plan", action="store_true",
                    help="skip the comparison leg whose refresh plan is made on the host before the timed region")
    ap.add_argument("--no-scaled-scoring", action="store_true",
                    help="skip the scaled-batch legs (cs_score_compact, block projection, residual proxy, "
                         "three-axis re-rotation)")
    ap.add_argument("--no-power-probe", action="store_true",
                    help="skip the legs that hold a load for a few seconds while sampling power and clock "
                         "(the matrix-core rate probe and the headline step)")
    ap.add_argument("--side-legs-workload", default="cfg2_qwen7b_32streams",
                    help="the workload whose shapes the side legs (scaled scoring, front end) use when "
                         "several workloads are measured")
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


def smi_sample():
    """Socket power (W) and graphics clock (MHz) from `amd-smi metric`, or None where the tool is
    missing or prints something else.  Reported beside the figures, never used in them."""
    import re
    import subprocess
    try:
        o = subprocess.run(["amd-smi", "metric", "--power", "--clock"], capture_output=True, text=True, timeout=15).stdout
        p = re.search(r"SOCKET_POWER:\s*(\d+)", o)
        c = re.search(r"GFX_0:\s*\n\s*CLK:\s*(\d+)", o)
        if p and c:
            return int(p.group(1)), int(c.group(1))
    except Exception:
        pass
    return None


def sampled_while(torch, enqueue, seconds):
    """Keeps the GPU busy with enqueue() for `seconds` and samples power / clock from a thread once
    the load has been on for a while; returns (samples, calls made, wall seconds)."""
    import threading
    samples, stop = [], []

    def sampler():
        time.sleep(min(1.0, seconds / 3))
        while not stop:
            v = smi_sample()
            if v:
                samples.append(v)
            time.sleep(0.3)
    th = threading.Thread(target=sampler)
    th.start()
    t0 = time.perf_counter()
    n = 0
    while time.perf_counter() - t0 < seconds:
        enqueue()
        torch.cuda.synchronize()
        n += 1
    wall = time.perf_counter() - t0
    stop.append(1)
    th.join()
    return samples, n, wall


def mfma_probe(torch, binding, seconds=1.5):
    """What the bf16 matrix cores of this device sustain with nothing else running: the library's
    probe kernel (register operands only) on 2 workgroups per CU, with constant and with
    pseudo-random operands, each held for `seconds` with power and clock sampled meanwhile."""
    n_wg, iters = 512, 200000
    sink = torch.zeros((n_wg * 256,), dtype=torch.float32, device="cuda")
    flops = n_wg * 4 * iters * 8 * 32768.0
    out = {}
    for label, rnd in (("constant_operands", 0), ("random_operands", 1)):
        binding.cs_mfma_rate_probe(sink, n_wg, 1000, rnd)
        torch.cuda.synchronize()
        samples, n, wall = sampled_while(torch, lambda: binding.cs_mfma_rate_probe(sink, n_wg, iters, rnd), seconds)
        ms = event_time(torch, lambda: binding.cs_mfma_rate_probe(sink, n_wg, iters, rnd), 2)
        out[label] = dict(TFLOPs=flops / ms / 1e9, frac_of_published_peak=flops / ms / 1e9 / PEAK_MFMA_BF16_TFLOPS,
                          socket_power_w=max([p for p, _ in samples], default=None),
                          gfx_clock_mhz=min([c for _, c in samples], default=None))
    return out


def graph_time(torch, run, steps, warmup):
    """Captures run() in a HIP graph (after one eager run on a side stream) and returns the wall
    milliseconds per replay over `steps` replays that follow `warmup` untimed ones."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for _ in range(warmup):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    return 1e3 * (time.perf_counter() - t0) / steps, graph


def host_route_time(w, data, step, torch):
    """Wall time of the host route that cs_plan_refresh replaces: copy the offsets back, plan on
    the host, copy the lists to the device (test-side planner; not part of any timed step)."""
    import numpy as np
    from paper_2604_06036_amd import planner

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
    return 1e3 * (time.perf_counter() - t0) / 5


def frontend_step(w, torch, engine, steps, warmup):
    """The chain from decoder output to attention output in one HIP graph: block projection,
    residual proxy, scoring with rescue, refresh plan on the GPU, position correction, then per
    layer refresh write + attention, on lists sized to the step's capacities (every token of a new
    frame may be kept).  Its executed-token count comes from the device plan."""
    data = engine.assemble_frontend_step(w, engine.hip_scorer, device="cuda")
    step = engine.FrontEndStep(data)
    step.run()
    torch.cuda.synchronize()
    totals = step.totals.cpu().tolist()
    if totals[2] != 0:
        raise RuntimeError(f"front-end step: plan flags {totals}")
    ms, _graph = graph_time(torch, step.run, steps, warmup)
    t_front = event_time(torch, step.front_end, max(3, min(steps, 20)))
    t_plan = event_time(torch, step.score_and_plan, max(3, min(steps, 20)))
    return dict(ms_per_step=ms, executed_tokens=totals[1], reused_rows=totals[0], q_cap=data.q_cap,
                tokens_per_s=totals[1] / (ms * 1e-3), front_end_ms=t_front, score_and_plan_ms=t_plan,
                frames=int(data.frame_type.shape[0]), blocks=int(data.blocks.shape[0]))


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(w, data, step, k_rows_before, pick, torch):
    """The oracle, as it stands, on the host: scoring of the step's frames, re-rotation of a sample
    of the reused rows (all layers), refresh write + attention of ONE layer on a sample of the
    executed rows, each scaled to the whole step; once on all host threads and once on one."""
    import numpy as np
    from oracle import codecsight_oracle as oc
    from threadpoolctl import threadpool_info, threadpool_limits
    all_threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    p = data.plan
    f64 = lambda t: t.detach().cpu().float().numpy().astype(np.float64)
    rows = int(p.src_slot.shape[0])
    n_q = int(p.q_pos.size)
    k_l, v_l = f64(step.k_pool[0]), f64(step.v_pool[0])          # cache of layer 0 after the step (not timed)
    kn, vn, q_l = f64(step.k_new[0][:n_q]), f64(step.v_new[0][:n_q]), f64(step.q[0][:n_q])
    k_host = k_rows_before.float().numpy().astype(np.float64)

    def timed(threads, max_q, max_rot):
        with threadpool_limits(limits=threads):
            t0 = time.perf_counter()
            oc.score_compact(data.mv, data.sad if w.use_residual else None, None, data.frame_type, data.cu_frames,
                             data.acc_in.copy(), w.grid_h, w.grid_w, w.group, w.tau_mv_sq, w.tau_sad, w.use_residual)
            t_a = time.perf_counter() - t0
            n_rot = min(max_rot, pick.size)
            t0 = time.perf_counter()
            if n_rot:
                oc.rotate(k_host[:, :n_rot], p.delta[pick[:n_rot]].astype(np.float64)[None, :, None], w.rope_base)
            t_b = (time.perf_counter() - t0) * rows / max(1, n_rot)
            t0 = time.perf_counter()
            oc.scatter(k_l, kn, p.q_slot)
            oc.scatter(v_l, vn, p.q_slot)
            t_c = time.perf_counter() - t0
            qrows = None if n_q <= max_q else np.sort(np.random.default_rng(1).choice(n_q, max_q, replace=False))
            t0 = time.perf_counter()
            oc.window_attn(q_l, k_l, v_l, p.cu_q, p.q_pos, p.layout.block_table, w.n_q_heads,
                           data.softmax_scale, rows=qrows)
            t_d = (time.perf_counter() - t0) * (1.0 if qrows is None else n_q / qrows.size)
        t_step = t_a + t_b + w.n_layers * (t_c + t_d)
        return dict(tokens_per_s=n_q / t_step, seconds_per_step=t_step, threads=int(threads),
                    parts_s=dict(score_compact=t_a, kv_rerotate=t_b, refresh_scatter_per_layer=t_c,
                                 attention_per_layer=t_d),
                    queries_sampled=int(min(n_q, max_q)), rotated_rows_sampled=int(min(max_rot, pick.size)))

    multi = timed(all_threads, 4096, 4096)
    single = timed(1, 512, 512)
    sample = (f"oracle (NumPy, fp64): scoring of the step's {data.frame_type.shape[0]} frames; re-rotation of "
              f"{multi['rotated_rows_sampled']} of {rows} reused rows x {w.n_layers} layers; refresh write of all "
              f"{n_q} rows and attention of {multi['queries_sampled']} of {n_q} executed rows for 1 of {w.n_layers} "
              f"layers; each part scaled to the whole step (single-thread leg: {single['queries_sampled']} queries, "
              f"{single['rotated_rows_sampled']} rows)")
    return dict(value=multi["tokens_per_s"], unit="tokens/s", cores=int(all_threads), kind="oracle", sample=sample,
                seconds_per_step=multi["seconds_per_step"], cpu_model=cpu_model(), host_cpus=os.cpu_count(),
                all_threads=multi, single_thread=single, workload=w.name)


def kernel_rooflines(w, work, t_a, t_plan, t_b, t_c, t_d, traffic_for):
    """Per-kernel figures of one workload: algorithmic bytes or flops per launch over the event-timed
    launch duration, against the published peak that bounds the kernel."""
    L = w.n_layers
    def hbm(name, kernel, ms, nbytes, launches):
        ach = nbytes / ms / 1e6
        t = traffic_for(name)
        return dict(kernel=kernel, bound="hbm", ms=ms, launches_per_step=launches, algorithmic_bytes=nbytes,
                    achieved=ach, peak=PEAK_HBM_GBS, unit="GB/s", frac=ach / PEAK_HBM_GBS, GBps=ach,
                    traffic=None if t is None else t["read_bytes"] + t["write_bytes"])
    out = {
        "cs_score_compact": hbm("cs_score_compact", "score_compact_kernel (+ clear_words_kernel)", t_a, work["a_bytes"], 1),
        "cs_plan_refresh": dict(kernel="plan_frames_kernel + plan_streams_kernel + plan_fill_kernel", bound="latency",
                                ms=t_plan, launches_per_step=1),
        "cs_kv_rerotate": hbm("cs_kv_rerotate", "rerotate_kernel", t_b, work["b_bytes"], 1),
        "cs_kv_refresh_scatter": hbm("cs_kv_refresh_scatter", "scatter_kernel", t_c, work["c_bytes"], L),
    }
    ach = work["d_flops"] / t_d / 1e9
    t = traffic_for("cs_window_prefill_attn")
    tm = traffic_for("attn_merge")
    traffic = None if t is None else t["read_bytes"] + t["write_bytes"] + (0 if tm is None else tm["read_bytes"] + tm["write_bytes"])
    name = ("window_attn_bf16_stream_kernel (+ window_attn_merge_kernel where the key sweep is split; the planning "
            "kernel runs once per step)" if w.dtype == "bf16" and w.head_dim == 128 else
            "window_attn_bf16_kernel" if w.dtype == "bf16" else "window_attn_f32_kernel")
    out["cs_window_prefill_attn"] = dict(kernel=name, bound="mfma", ms=t_d, launches_per_step=L,
                                         flops_per_launch=work["d_flops"], algorithmic_bytes=work["d_bytes"],
                                         achieved=ach, peak=PEAK_MFMA_BF16_TFLOPS, unit="TFLOP/s",
                                         frac=ach / PEAK_MFMA_BF16_TFLOPS, TFLOPs=ach,
                                         GBps=work["d_bytes"] / t_d / 1e6, traffic=traffic)
    return out


def measure_workload(w, args, torch, binding, engine, keep_for_cpu, probe_power=False):
    """One workload: the device-planned step in a HIP graph (the figure that counts), the
    host-planned step beside it, event-timed launches of every call, and their rooflines."""
    import numpy as np
    t_setup = time.perf_counter()
    data = engine.assemble_step(w, engine.hip_scorer, device="cuda")
    info = data.info
    cap = lambda n: (n + n // 8 + 255) // 256 * 256
    step = engine.DeviceStep(data, reuse_cap=cap(info["n_reuse"]), q_cap=cap(info["n_q"]),
                             overlap=False if args.no_overlap else None)
    cpu_inputs = None
    if keep_for_cpu:                       # a sample of the pre-step cache rows for the oracle's re-rotation leg
        rows = int(data.plan.src_slot.shape[0])
        pick = np.arange(rows) if rows <= 4096 else np.sort(np.random.default_rng(0).choice(rows, 4096, replace=False))
        idx = torch.from_numpy(data.plan.src_slot[pick].astype(np.int64)).to(step.dev)
        cpu_inputs = (step.k_pool[:, idx].cpu(), pick)
    print(f"[bench] {w.name}: {info} setup {time.perf_counter() - t_setup:.1f}s", file=sys.stderr, flush=True)

    launch = "eager" if args.eager else "hipgraph"
    if args.eager:
        for _ in range(args.warmup):
            step.run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step.run()
        torch.cuda.synchronize()
        ms_per_step = 1e3 * (time.perf_counter() - t0) / args.steps
    else:
        ms_per_step, _graph = graph_time(torch, step.run, args.steps, args.warmup)
    sustained = None
    if probe_power and not args.eager:
        # the same graph replayed back to back for a few seconds, power and clock sampled meanwhile
        samples, n, wall = sampled_while(torch, lambda: [_graph.replay() for _ in range(10)], 3.0)
        sustained = dict(ms_per_step=1e3 * wall / (10 * n), seconds=wall,
                         socket_power_w=max([p for p, _ in samples], default=None),
                         gfx_clock_mhz=min([c for _, c in samples], default=None))
    totals = step.totals.cpu().tolist()
    if totals != [info["n_reuse"], info["n_q"], 0, 0]:
        raise RuntimeError(f"device plan totals {totals} differ from the generator's {info['n_reuse']}, {info['n_q']}")
    status = step.scoring_status()
    if status != 0:
        raise RuntimeError(f"cs_score_compact: look-back wait timed out (status word {status})")
    # visible (query, key) pairs of the step, from the plan the GPU made
    info["visible_pairs"] = float((step.q_pos[: info["n_q"]].to(torch.int64) + 1).sum().item())
    work = kernel_bytes_flops(w, info, w.n_layers)

    # ---- per-kernel clocks: HIP events on the launch stream around back-to-back launches
    L = w.n_layers
    reps = max(3, min(args.steps, 20))
    t_a = event_time(torch, step.score_compact, reps)
    t_plan = event_time(torch, step.plan_refresh, reps)
    t_b = event_time(torch, step.rerotate, reps)
    t_c = event_time(torch, lambda: [step.refresh_scatter(l) for l in range(L)], reps) / L
    t_d = event_time(torch, lambda: [step.attention(l, reuse_plan=l > 0) for l in range(L)], reps) / L

    # HBM bytes per launch from committed rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this same
    # command (profiles/), calibrated against a plain copy: not measured live; stamped with the
    # commit the counters were taken at; null where no such run exists for the workload
    per_wl, traffic_commit = {}, None
    tpath = os.path.join(ROOT, "profiles", "pmc_traffic.json")
    if os.path.exists(tpath):
        try:
            doc = json.load(open(tpath))
            per_wl = doc.get(w.name, {})
            traffic_commit = doc.get("_commit")
        except Exception:
            per_wl = {}
    kernels = kernel_rooflines(w, work, t_a, t_plan, t_b, t_c, t_d, lambda name: per_wl.get(name))
    share = {k: v["ms"] * v["launches_per_step"] for k, v in kernels.items()}
    dominant = max(share, key=share.get)
    roofline = dict(kernels[dominant])
    roofline["call"] = dominant
    roofline["ms_per_launch"] = roofline.pop("ms")
    roofline["traffic_source"] = (None if roofline.get("traffic") is None else
                                  f"profiles/pmc_traffic.json (rocprofv3 --pmc, taken at commit {traffic_commit})")
    res = dict(workload=w.name, ms_per_step=ms_per_step, tokens_per_s=info["n_q"] / (ms_per_step * 1e-3),
               window_tokens_per_s=info["kv_len_total"] / (ms_per_step * 1e-3), launch=launch, dtype=w.dtype,
               streams=w.n_streams, layers=L, heads=f"{w.n_q_heads}/{w.n_kv_heads}", head_dim=w.head_dim,
               window_frames=w.window, stride_frames=w.stride, tokens_per_frame=w.tokens_per_frame,
               executed_tokens=info["n_q"], reused_rows=info["n_reuse"], window_tokens=info["kv_len_total"],
               reuse_cap=step.reuse_cap, q_cap=step.q_cap, kernels=kernels, roofline=roofline,
               kernel_ms_sum=sum(share.values()))
    if sustained:
        res["sustained"] = sustained
    res["rerotate_schedule"] = (f"second stream beside the layer loop, {step.layers_per_rerotate} layers per call"
                                if step.overlap else "one call ahead of the layer loop")
    if step.overlap and not args.eager:
        # the same step with the position correction as one call ahead of the layer loop
        sstep = engine.DeviceStep(data, reuse_cap=step.reuse_cap, q_cap=step.q_cap, overlap=False)
        res["serial_ms_per_step"], _g4 = graph_time(torch, sstep.run, args.steps, args.warmup)
        del _g4, sstep
    if not args.no_fused_step and not args.eager:
        # the same step with each layer's refresh write inside the attention launch (one call per
        # layer instead of two); reported beside the default route, which stays the one that is faster
        fstep = engine.DeviceStep(data, reuse_cap=step.reuse_cap, q_cap=step.q_cap, fused=True, overlap=False)
        res["fused_ms_per_step"], _g3 = graph_time(torch, fstep.run, args.steps, args.warmup)
        del _g3
        if fstep.attention_status() != 0:
            raise RuntimeError("cs_refresh_prefill_attn: the launch-wide wait ran into its bound")
        t_f = event_time(torch, lambda: [fstep.refresh_and_attention(l, reuse_plan=l > 0) for l in range(L)], reps) / L
        res["fused_call_ms"] = t_f
        res["separate_calls_ms"] = t_c + t_d
        del fstep
    if not args.no_host_plan:
        hstep = engine.DeviceStep(data, host_plan=True, overlap=step.overlap)
        if args.eager:
            hstep.run(); torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                hstep.run()
            torch.cuda.synchronize()
            res["host_planned_ms_per_step"] = 1e3 * (time.perf_counter() - t0) / args.steps
        else:
            res["host_planned_ms_per_step"], _g2 = graph_time(torch, hstep.run, args.steps, args.warmup)
            del _g2
        res["host_route_ms"] = host_route_time(w, data, step, torch)
        del hstep
    return res, data, step, cpu_inputs, work


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the path shards by stream with no exchange step; "
              "no multi-GPU figure is produced). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
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
    names = [args.workload] if args.workload else list(DEFAULT_WORKLOADS)
    headline = names[-1]
    side_name = args.side_legs_workload if (len(names) > 1 and args.side_legs_workload in names) else headline
    results, side, cpu = [], {}, None
    for name in names:
        w = synth.WORKLOADS[name]
        res, data, step, cpu_inputs, work = measure_workload(w, args, torch, binding, engine,
                                                             keep_for_cpu=(name == headline and not args.no_cpu_baseline),
                                                             probe_power=(name == headline and not args.no_power_probe))
        results.append(res)
        reps = max(3, min(args.steps, 20))
        if name == side_name:
            if not args.no_scaled_scoring:
                side["score_compact_scaled"] = scaled_scoring(w, torch, binding)
                side["block_projection"] = block_projection(w, torch, binding, reps)
                side["residual_proxy"] = residual_proxy(w, torch, binding, reps)
                side["kv_rerotate_axes"] = axes_rerotation(w, step, torch, binding, work["b_bytes"], reps)
            if not args.no_frontend_step:
                side["frontend_step"] = frontend_step(w, torch, engine, args.steps, args.warmup)
            side["side_legs_workload"] = name
        if cpu_inputs is not None:
            cpu = cpu_baseline(w, data, step, cpu_inputs[0], cpu_inputs[1], torch)
        del data, step, cpu_inputs
        torch.cuda.empty_cache()

    head = results[-1]
    out = {
        "metric": "window-prefill tokens/s per MI355X (executed refresh+new+text tokens per second, whole step "
                  "with the refresh plan made on the GPU)",
        "value": head["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": head["dtype"],
        "data": "synthetic",
        "config": {"workload": head["workload"], "streams": head["streams"], "layers": head["layers"],
                   "heads": head["heads"], "head_dim": head["head_dim"], "window_frames": head["window_frames"],
                   "stride_frames": head["stride_frames"], "tokens_per_frame": head["tokens_per_frame"],
                   "executed_tokens": head["executed_tokens"], "reused_rows": head["reused_rows"],
                   "window_tokens": head["window_tokens"], "launch": head["launch"],
                   "plan": "device (cs_plan_refresh inside the step)",
                   "rerotate_schedule": head["rerotate_schedule"]},
        "window_tokens_per_s": head["window_tokens_per_s"],
        "kernels": head["kernels"],
        "roofline": head["roofline"],
        "workloads": results,
    }
    if args.calibrate_copy:
        out["copy_calibration"] = copy_calibration(torch)
    if not args.no_power_probe:
        out["mfma_probe"] = mfma_probe(torch, binding)
        if "sustained" in head:
            out["sustained_headline_step"] = head["sustained"]
    out.update(side)
    if cpu is not None:
        out["cpu_baseline"] = cpu
    print(json.dumps(out))


if __name__ == "__main__":
    main()
