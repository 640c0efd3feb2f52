"""Thin ctypes binding over libcodecsight.so: argument marshalling only.

Every function has the name and argument order of its C entry point (include/codecsight.h) and
takes torch tensors that already live on the GPU; the work is enqueued on torch's current stream.
Nothing here computes anything, and there is no fallback: a missing library is an ImportError at
first use, and a non-zero status code raises CodecSightError.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcodecsight.so")

CS_OK, CS_EINVAL, CS_EUNSUPPORTED, CS_EHIP, CS_EWORKSPACE = 0, -1, -2, -3, -4
CS_F32, CS_BF16 = 0, 1
CS_ATTN_PLAN_BUILD, CS_ATTN_PLAN_REUSE, CS_ATTN_PLAN_ONLY = 0, 1, 2
CS_FRAME_P, CS_FRAME_I = 0, 1
CS_ROPE_HALF_SPLIT, CS_ROPE_INTERLEAVED = 0, 1
CS_KV_BLOCK = 16

_ERR = {CS_EINVAL: "CS_EINVAL", CS_EUNSUPPORTED: "CS_EUNSUPPORTED", CS_EHIP: "CS_EHIP",
        CS_EWORKSPACE: "CS_EWORKSPACE"}

EXPORTS = ("cs_version", "cs_last_hip_error", "cs_mfma_rate_probe", "cs_project_blocks", "cs_residual_proxy", "cs_score_compact_workspace", "cs_score_compact",
           "cs_score_compact_noalloc",
           "cs_plan_refresh_workspace", "cs_plan_refresh", "cs_kv_rerotate", "cs_kv_rerotate_axes", "cs_kv_refresh_scatter",
           "cs_window_prefill_attn_workspace",
           "cs_window_prefill_attn", "cs_refresh_prefill_attn")


class CodecSightError(RuntimeError):
    def __init__(self, fn: str, code: int, hip: int = 0):
        self.code = code
        self.hip = hip
        extra = f" (hipError {hip})" if code == CS_EHIP else ""
        super().__init__(f"{fn} failed: {_ERR.get(code, code)}{extra}")


_lib = None


def lib() -> ctypes.CDLL:
    """Opens the HIP library (built by `python -m paper_2604_06036_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_06036_amd.build`; "
                          "there is no CPU fallback")
    L = ctypes.CDLL(LIB_PATH)
    c = ctypes
    vp, i32, i64, u32, sz, f32 = c.c_void_p, c.c_int32, c.c_int64, c.c_uint32, c.c_size_t, c.c_float
    L.cs_version.restype = c.c_char_p
    L.cs_version.argtypes = []
    L.cs_last_hip_error.restype = c.c_int
    L.cs_last_hip_error.argtypes = []
    L.cs_score_compact_workspace.restype = sz
    L.cs_score_compact_workspace.argtypes = [i32, i32, i32, i32, i32]
    L.cs_score_compact.restype = c.c_int
    L.cs_score_compact.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, u32, u32, i32,
                                   vp, vp, vp, vp, sz, vp]
    L.cs_score_compact_noalloc.restype = c.c_int
    L.cs_score_compact_noalloc.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, u32, u32, i32,
                                           vp, vp, vp, vp]
    L.cs_mfma_rate_probe.restype = c.c_int
    L.cs_mfma_rate_probe.argtypes = [vp, i32, i32, i32, vp]
    L.cs_project_blocks.restype = c.c_int
    L.cs_project_blocks.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp]
    L.cs_residual_proxy.restype = c.c_int
    L.cs_residual_proxy.argtypes = [vp, vp, vp, i32, i32, i32, i64, i64, i32, i32, i32, i32, i32, i32, vp, vp]
    L.cs_plan_refresh_workspace.restype = sz
    L.cs_plan_refresh_workspace.argtypes = [i32, i32]
    L.cs_plan_refresh.restype = c.c_int
    L.cs_plan_refresh.argtypes = [vp, vp, vp, vp, vp, i32, vp, i32, i32, i32, i32, i32, i32, i64, i64,
                                  vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.cs_kv_rerotate.restype = c.c_int
    L.cs_kv_rerotate.argtypes = [vp, vp, vp, vp, vp, i64, i32, i32, i32, i64, i64, i64, f32, i32, i32, vp]
    L.cs_kv_rerotate_axes.restype = c.c_int
    L.cs_kv_rerotate_axes.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, i64, i64, i64, f32, i32, i32, vp]
    L.cs_kv_refresh_scatter.restype = c.c_int
    L.cs_kv_refresh_scatter.argtypes = [vp, vp, vp, vp, vp, i64, i32, i32, i64, i64, i32, vp]
    L.cs_window_prefill_attn_workspace.restype = sz
    L.cs_window_prefill_attn_workspace.argtypes = [i64, i32, i32, i32, i32, i32, i32]
    L.cs_window_prefill_attn.restype = c.c_int
    L.cs_window_prefill_attn.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, i64, i32, i32, i32,
                                         i32, i64, i64, f32, i32, vp, sz, i32, vp]
    L.cs_refresh_prefill_attn.restype = c.c_int
    L.cs_refresh_prefill_attn.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, i64, i32, i32, i32,
                                          i32, i64, i64, f32, i32, vp, sz, i32, vp]
    _lib = L
    return L


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _need(fn: str, t: Optional[torch.Tensor], n: int, what: str):
    """Marshalling guard: an index / data tensor shorter than the count passed beside it would make
    the kernel read past its end, so it is refused here."""
    if t is not None and t.numel() < n:
        raise ValueError(f"{fn}: {what} holds {t.numel()} elements, {n} needed")


def _check(fn: str, code: int):
    if code != CS_OK:
        raise CodecSightError(fn, code, lib().cs_last_hip_error() if code == CS_EHIP else 0)


def dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return CS_F32
    if t.dtype == torch.bfloat16:
        return CS_BF16
    raise CodecSightError("dtype", CS_EUNSUPPORTED)


def cs_version() -> str:
    return lib().cs_version().decode()


def cs_mfma_rate_probe(sink, n_workgroups, iters, random_operands):
    _need("cs_mfma_rate_probe", sink, n_workgroups * 256, "sink")
    _check("cs_mfma_rate_probe", lib().cs_mfma_rate_probe(_ptr(sink), n_workgroups, iters, int(bool(random_operands)), _stream()))


def cs_score_compact_workspace(n_streams, n_frames, grid_h, grid_w, group) -> int:
    return int(lib().cs_score_compact_workspace(n_streams, n_frames, grid_h, grid_w, group))


def cs_score_compact(mv, sad, intra, frame_type, cu_frames, acc_mask, n_streams, n_frames, grid_h,
                     grid_w, group, tau_mv_sq, tau_sad, use_residual, keep_mask, kept_idx, kept_off,
                     workspace, workspace_bytes=None):
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    fn = "cs_score_compact"
    n_patch, n_tok = grid_h * grid_w, (grid_h // max(1, group)) * (grid_w // max(1, group))
    _need(fn, mv, n_frames * n_patch * 2, "mv"); _need(fn, sad, n_frames * n_patch, "sad")
    _need(fn, intra, n_frames * n_patch, "intra"); _need(fn, frame_type, n_frames, "frame_type")
    _need(fn, cu_frames, n_streams + 1, "cu_frames"); _need(fn, acc_mask, n_streams * n_patch, "acc_mask")
    _need(fn, keep_mask, n_frames * n_tok, "keep_mask"); _need(fn, kept_idx, n_frames * n_tok, "kept_idx")
    _need(fn, kept_off, n_frames + 1, "kept_off")
    if workspace is not None and workspace.numel() * workspace.element_size() < workspace_bytes:
        raise ValueError("cs_score_compact: workspace tensor smaller than workspace_bytes")
    _check("cs_score_compact", lib().cs_score_compact(
        _ptr(mv), _ptr(sad), _ptr(intra), _ptr(frame_type), _ptr(cu_frames), _ptr(acc_mask),
        n_streams, n_frames, grid_h, grid_w, group, tau_mv_sq, tau_sad, int(bool(use_residual)),
        _ptr(keep_mask), _ptr(kept_idx), _ptr(kept_off), _ptr(workspace), workspace_bytes, _stream()))


def cs_score_compact_noalloc(mv, sad, intra, frame_type, cu_frames, acc_mask, n_streams, n_frames, grid_h,
                             grid_w, group, tau_mv_sq, tau_sad, use_residual, keep_mask, kept_idx, kept_off):
    fn = "cs_score_compact_noalloc"
    n_patch, n_tok = grid_h * grid_w, (grid_h // max(1, group)) * (grid_w // max(1, group))
    _need(fn, mv, n_frames * n_patch * 2, "mv"); _need(fn, sad, n_frames * n_patch, "sad")
    _need(fn, intra, n_frames * n_patch, "intra"); _need(fn, frame_type, n_frames, "frame_type")
    _need(fn, cu_frames, n_streams + 1, "cu_frames"); _need(fn, acc_mask, n_streams * n_patch, "acc_mask")
    _need(fn, keep_mask, n_frames * n_tok, "keep_mask"); _need(fn, kept_idx, n_frames * n_tok, "kept_idx")
    _need(fn, kept_off, n_frames + 1, "kept_off")
    _check(fn, lib().cs_score_compact_noalloc(
        _ptr(mv), _ptr(sad), _ptr(intra), _ptr(frame_type), _ptr(cu_frames), _ptr(acc_mask),
        n_streams, n_frames, grid_h, grid_w, group, tau_mv_sq, tau_sad, int(bool(use_residual)),
        _ptr(keep_mask), _ptr(kept_idx), _ptr(kept_off), _stream()))


CS_SCORE_STATUS_OFFSET = 4


def cs_score_compact_status(workspace, workspace_bytes=None) -> int:
    """The device status word cs_score_compact leaves in its workspace (0 = good).  The caller
    synchronises first; this only copies the word back."""
    if workspace is None or workspace.numel() * workspace.element_size() < CS_SCORE_STATUS_OFFSET + 4:
        return 0
    flat = workspace.view(-1).view(__import__("torch").uint8)
    return int(flat[CS_SCORE_STATUS_OFFSET:CS_SCORE_STATUS_OFFSET + 4].view(__import__("torch").int32).item())


def cs_kv_rerotate(k_cache, v_cache, src_slot, dst_slot, delta, n_rows, n_layers, n_kv_heads, head_dim,
                   stride_layer, stride_slot, stride_head, rope_base, rope_style, dtype):
    for t, what in ((src_slot, "src_slot"), (dst_slot, "dst_slot"), (delta, "delta")):
        _need("cs_kv_rerotate", t, n_rows, what)
    _check("cs_kv_rerotate", lib().cs_kv_rerotate(
        _ptr(k_cache), _ptr(v_cache), _ptr(src_slot), _ptr(dst_slot), _ptr(delta), n_rows, n_layers,
        n_kv_heads, head_dim, stride_layer, stride_slot, stride_head, rope_base, rope_style, dtype,
        _stream()))


def cs_project_blocks(blocks, cu_blocks, n_frames, src_w, src_h, in_w, in_h, patch, grid_h, grid_w, mv, intra,
                      n_blocks=None):
    """blocks: uint8 / int32 tensor holding the 16-byte records; n_blocks (= cu_blocks[-1], known to the
    caller) only serves the length check."""
    fn = "cs_project_blocks"
    _need(fn, cu_blocks, n_frames + 1, "cu_blocks")
    if n_blocks is not None and blocks is not None and blocks.numel() * blocks.element_size() < 16 * n_blocks:
        raise ValueError(f"{fn}: blocks holds fewer than {n_blocks} records")
    if grid_h > 0 and grid_w > 0:
        _need(fn, mv, n_frames * grid_h * grid_w * 2, "mv"); _need(fn, intra, n_frames * grid_h * grid_w, "intra")
    _check(fn, lib().cs_project_blocks(_ptr(blocks), _ptr(cu_blocks), n_frames, src_w, src_h, in_w, in_h, patch,
                                       grid_h, grid_w, _ptr(mv), _ptr(intra), _stream()))


def cs_residual_proxy(cur, prev, mv_field, n_frames, src_w, src_h, pitch, frame_stride, cell, in_w, in_h, patch,
                      grid_h, grid_w, res):
    fn = "cs_residual_proxy"
    if n_frames > 0 and cell > 0:
        _need(fn, cur, n_frames * frame_stride, "cur"); _need(fn, prev, n_frames * frame_stride, "prev")
        _need(fn, mv_field, n_frames * (-(-src_h // cell)) * (-(-src_w // cell)) * 2, "mv_field")
        _need(fn, res, n_frames * grid_h * grid_w, "res")
    _check(fn, lib().cs_residual_proxy(_ptr(cur), _ptr(prev), _ptr(mv_field), n_frames, src_w, src_h, pitch,
                                       frame_stride, cell, in_w, in_h, patch, grid_h, grid_w, _ptr(res), _stream()))


def cs_plan_refresh_workspace(n_streams, window) -> int:
    return int(lib().cs_plan_refresh_workspace(n_streams, window))


def cs_plan_refresh(old_types, old_counts, new_types, kept_off, block_table_old, max_blocks_old,
                    block_table_new, max_blocks_new, n_streams, window, stride, n_text, tokens_per_frame,
                    reuse_cap, q_cap, src_slot, dst_slot, delta, q_pos, q_slot, q_kind, cu_q, kv_len,
                    out_types, out_counts, totals, workspace, workspace_bytes=None):
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    fn = "cs_plan_refresh"
    if n_streams > 0 and window > 0 and 0 < stride <= window:
        _need(fn, old_types, n_streams * window, "old_types"); _need(fn, old_counts, n_streams * window, "old_counts")
        _need(fn, new_types, n_streams * stride, "new_types"); _need(fn, kept_off, n_streams * stride + 1, "kept_off")
        _need(fn, block_table_old, n_streams * max_blocks_old, "block_table_old")
        _need(fn, block_table_new, n_streams * max_blocks_new, "block_table_new")
        _need(fn, out_types, n_streams * window, "out_types"); _need(fn, out_counts, n_streams * window, "out_counts")
        _need(fn, cu_q, n_streams + 1, "cu_q"); _need(fn, kv_len, n_streams, "kv_len")
    for t, what in ((src_slot, "src_slot"), (dst_slot, "dst_slot"), (delta, "delta")):
        _need(fn, t, reuse_cap, what)
    for t, what in ((q_pos, "q_pos"), (q_slot, "q_slot"), (q_kind, "q_kind")):
        _need(fn, t, q_cap, what)
    _need(fn, totals, 4, "totals")
    _check(fn, lib().cs_plan_refresh(
        _ptr(old_types), _ptr(old_counts), _ptr(new_types), _ptr(kept_off), _ptr(block_table_old), max_blocks_old,
        _ptr(block_table_new), max_blocks_new, n_streams, window, stride, n_text, tokens_per_frame, reuse_cap,
        q_cap, _ptr(src_slot), _ptr(dst_slot), _ptr(delta), _ptr(q_pos), _ptr(q_slot), _ptr(q_kind), _ptr(cu_q),
        _ptr(kv_len), _ptr(out_types), _ptr(out_counts), _ptr(totals), _ptr(workspace), workspace_bytes,
        _stream()))


def cs_kv_rerotate_axes(k_cache, v_cache, src_slot, dst_slot, delta3, axis_of_pair, n_rows, n_layers, n_kv_heads,
                        head_dim, stride_layer, stride_slot, stride_head, rope_base, rope_style, dtype):
    fn = "cs_kv_rerotate_axes"
    _need(fn, src_slot, n_rows, "src_slot"); _need(fn, dst_slot, n_rows, "dst_slot")
    _need(fn, delta3, 3 * n_rows, "delta3"); _need(fn, axis_of_pair, head_dim // 2, "axis_of_pair")
    _check(fn, lib().cs_kv_rerotate_axes(
        _ptr(k_cache), _ptr(v_cache), _ptr(src_slot), _ptr(dst_slot), _ptr(delta3), _ptr(axis_of_pair), n_rows,
        n_layers, n_kv_heads, head_dim, stride_layer, stride_slot, stride_head, rope_base, rope_style, dtype,
        _stream()))


def cs_kv_refresh_scatter(k_new, v_new, slot, k_cache_layer, v_cache_layer, n_tok, n_kv_heads, head_dim,
                          stride_slot, stride_head, dtype):
    fn = "cs_kv_refresh_scatter"
    _need(fn, slot, n_tok, "slot"); _need(fn, k_new, n_tok * n_kv_heads * head_dim, "k_new")
    _need(fn, v_new, n_tok * n_kv_heads * head_dim, "v_new")
    _check("cs_kv_refresh_scatter", lib().cs_kv_refresh_scatter(
        _ptr(k_new), _ptr(v_new), _ptr(slot), _ptr(k_cache_layer), _ptr(v_cache_layer), n_tok,
        n_kv_heads, head_dim, stride_slot, stride_head, dtype, _stream()))


def cs_window_prefill_attn_workspace(n_q, n_streams, n_q_heads, n_kv_heads, head_dim, max_blocks, dtype) -> int:
    return int(lib().cs_window_prefill_attn_workspace(n_q, n_streams, n_q_heads, n_kv_heads, head_dim,
                                                      max_blocks, dtype))


def cs_window_prefill_attn(q, k_cache_layer, v_cache_layer, cu_q, q_pos, kv_len, block_table, max_blocks,
                           block_size, out, n_q, n_streams, n_q_heads, n_kv_heads, head_dim, stride_slot,
                           stride_head, softmax_scale, dtype, workspace=None, workspace_bytes=None,
                           plan_mode=CS_ATTN_PLAN_BUILD):
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    fn = "cs_window_prefill_attn"
    _need(fn, q, n_q * n_q_heads * head_dim, "q"); _need(fn, out, n_q * n_q_heads * head_dim, "out")
    _need(fn, cu_q, n_streams + 1, "cu_q"); _need(fn, q_pos, n_q, "q_pos"); _need(fn, kv_len, n_streams, "kv_len")
    _need(fn, block_table, n_streams * max_blocks, "block_table")
    if workspace is not None and workspace.numel() * workspace.element_size() < workspace_bytes:
        raise ValueError("cs_window_prefill_attn: workspace tensor smaller than workspace_bytes")
    _check("cs_window_prefill_attn", lib().cs_window_prefill_attn(
        _ptr(q), _ptr(k_cache_layer), _ptr(v_cache_layer), _ptr(cu_q), _ptr(q_pos), _ptr(kv_len),
        _ptr(block_table), max_blocks, block_size, _ptr(out), n_q, n_streams, n_q_heads, n_kv_heads,
        head_dim, stride_slot, stride_head, softmax_scale, dtype, _ptr(workspace), workspace_bytes,
        plan_mode, _stream()))


CS_ATTN_STATUS_OFFSET = 56


def cs_refresh_prefill_attn(k_new, v_new, slot, n_tok, q, k_cache_layer, v_cache_layer, cu_q, q_pos, kv_len,
                            block_table, max_blocks, block_size, out, n_q, n_streams, n_q_heads, n_kv_heads,
                            head_dim, stride_slot, stride_head, softmax_scale, dtype, workspace=None,
                            workspace_bytes=None, plan_mode=CS_ATTN_PLAN_BUILD):
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    fn = "cs_refresh_prefill_attn"
    _need(fn, k_new, n_tok * n_kv_heads * head_dim, "k_new"); _need(fn, v_new, n_tok * n_kv_heads * head_dim, "v_new")
    _need(fn, slot, n_tok, "slot")
    _need(fn, q, n_q * n_q_heads * head_dim, "q"); _need(fn, out, n_q * n_q_heads * head_dim, "out")
    _need(fn, cu_q, n_streams + 1, "cu_q"); _need(fn, q_pos, n_q, "q_pos"); _need(fn, kv_len, n_streams, "kv_len")
    _need(fn, block_table, n_streams * max_blocks, "block_table")
    if workspace is not None and workspace.numel() * workspace.element_size() < workspace_bytes:
        raise ValueError(f"{fn}: workspace tensor smaller than workspace_bytes")
    _check(fn, lib().cs_refresh_prefill_attn(
        _ptr(k_new), _ptr(v_new), _ptr(slot), n_tok, _ptr(q), _ptr(k_cache_layer), _ptr(v_cache_layer), _ptr(cu_q),
        _ptr(q_pos), _ptr(kv_len), _ptr(block_table), max_blocks, block_size, _ptr(out), n_q, n_streams, n_q_heads,
        n_kv_heads, head_dim, stride_slot, stride_head, softmax_scale, dtype, _ptr(workspace), workspace_bytes,
        plan_mode, _stream()))


def cs_attn_status(workspace) -> int:
    """The barrier status word cs_refresh_prefill_attn leaves in the attention workspace (0 = good).
    The caller synchronises first; this only copies the word back."""
    if workspace is None or workspace.numel() * workspace.element_size() < CS_ATTN_STATUS_OFFSET + 4:
        return 0
    flat = workspace.view(-1).view(torch.uint8)
    return int(flat[CS_ATTN_STATUS_OFFSET:CS_ATTN_STATUS_OFFSET + 4].view(torch.int32).item())
