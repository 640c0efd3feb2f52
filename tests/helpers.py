"""Shared test helpers: oracle adapters and the tolerance checks of the parity bar."""
from __future__ import annotations

import numpy as np
import torch

from oracle import codecsight_oracle as oc


def oracle_scorer(mv, sad, frame_type, cu_frames, acc, w, tau_mv_sq, tau_sad):
    """Adapter with the scorer signature of engine.assemble_step, backed by the CPU oracle."""
    return oc.score_compact(mv, sad if w.use_residual else None, None, frame_type, cu_frames, acc,
                            w.grid_h, w.grid_w, w.group, tau_mv_sq, tau_sad, w.use_residual)


def f64(t) -> np.ndarray:
    """Exact widening of a torch tensor (fp32 or bf16) to float64 NumPy."""
    if isinstance(t, np.ndarray):
        return t.astype(np.float64)
    return t.detach().cpu().to(torch.float32).numpy().astype(np.float64)


def round_like(x64: np.ndarray, dtype: torch.dtype) -> torch.Tensor:
    """Round float64 values to the storage dtype (round to nearest even)."""
    return torch.from_numpy(np.ascontiguousarray(x64)).to(torch.float32).to(dtype)


def bf16_ulp_distance(a: torch.Tensor, b: torch.Tensor) -> np.ndarray:
    """Distance in bf16 units in the last place between two bf16 tensors (finite values)."""
    def key(t):
        bits = t.detach().cpu().contiguous().view(torch.int16).numpy().astype(np.int32) & 0xFFFF
        return np.where(bits & 0x8000, 0x8000 - bits, bits)      # monotone integer line
    return np.abs(key(a) - key(b))


def check_rerotated(gpu: torch.Tensor, ref64: np.ndarray, dtype: str):
    """The bar for re-rotated keys: 1e-2 max-abs against the un-rounded oracle (unit-scale data).

    bf16 storage rounds by up to 2^-9 |x|, which alone exceeds 1e-2 once |x| >= 5.12, so three
    things are checked: (i) the strict bound where rounding cannot break it (|ref| < 2.56),
    (ii) everywhere max(1e-2, half-ulp + 1e-5), (iii) the result is the correctly rounded oracle
    value or its bf16 neighbour -- except where the result nearly cancels (x_a cos ~ x_b sin): there
    the fp32 products of unit-scale operands carry ~1e-7 of noise, which is many ulps of a tiny
    result, so elements already within 2^-20 of the oracle are exempt from the ulp count.
    fp32 storage must hold 1e-5.
    """
    got = f64(gpu)
    err = np.abs(got - ref64)
    if dtype == "f32":
        assert err.max() <= 1e-5, err.max()
        return dict(max_abs=float(err.max()))
    small = np.abs(ref64) < 2.56
    assert err[small].max(initial=0.0) <= 1e-2
    assert np.all(err <= np.maximum(1e-2, 2.0 ** -8 * np.abs(ref64) + 1e-5))
    ulp = bf16_ulp_distance(gpu, round_like(ref64, torch.bfloat16))
    ulp = np.where(err <= 2.0 ** -20, 0, ulp)
    assert ulp.max(initial=0) <= 1, ulp.max()
    return dict(max_abs=float(err.max()), one_ulp_fraction=float((ulp == 1).mean()))


def check_attention(gpu: torch.Tensor, ref64: np.ndarray, dtype: str):
    """The bar for attention outputs: 2e-2 max-abs and 1e-2 mean-relative (mean|err| / mean|ref|)."""
    got = f64(gpu)
    assert np.isfinite(got).all()
    err = np.abs(got - ref64)
    max_abs = float(err.max(initial=0.0))
    mean_rel = float(err.mean() / max(np.abs(ref64).mean(), 1e-30)) if err.size else 0.0
    if dtype == "f32":
        assert max_abs <= 2e-5 and mean_rel <= 1e-5, (max_abs, mean_rel)
    else:
        assert max_abs <= 2e-2 and mean_rel <= 1e-2, (max_abs, mean_rel)
    return dict(max_abs=max_abs, mean_rel=mean_rel)


class OraclePlan:
    """The row lists of a step as the plan ORACLE makes them (token loops in oracle/plan_oracle.py),
    as NumPy arrays under the names the kernels' arguments have."""

    def __init__(self, data):
        from oracle import plan_oracle as po
        w, old, new = data.workload, data.old_layout, data.new_layout
        first_new = w.window - w.stride
        d = po.plan_batch(old.frame_type.tolist(), old.counts.tolist(), new.frame_type[:, first_new:].tolist(),
                          new.counts[:, first_new:].tolist(), w.n_text, w.tokens_per_frame,
                          old.block_table, new.block_table)
        i32 = lambda a: np.asarray(a, dtype=np.int32)
        self.src_slot, self.dst_slot, self.delta = i32(d["src_slot"]), i32(d["dst_slot"]), i32(d["delta"])
        self.q_pos, self.q_slot = i32(d["q_pos"]), i32(d["q_slot"])
        self.q_kind = np.asarray(d["q_kind"], dtype=np.uint8)
        self.cu_q, self.kv_len = i32(d["cu_q"]), i32(d["kv_len"])
        self.block_table = new.block_table


def assert_device_plan(step, plan: "OraclePlan"):
    """The lists cs_plan_refresh wrote for `step` equal the plan oracle's, entry for entry; list
    tails up to the capacities hold the padding values."""
    n_r, n_e = plan.src_slot.size, plan.q_pos.size
    assert step.totals.cpu().tolist() == [n_r, n_e, 0, 0], step.totals.cpu().tolist()
    for name in ("src_slot", "dst_slot", "delta"):
        got = getattr(step, name).cpu().numpy()
        assert np.array_equal(got[:n_r], getattr(plan, name)), name
        if step.reuse_cap > n_r:
            assert np.all(got[n_r:step.reuse_cap] == (0 if name == "delta" else -1)), name
    for name in ("q_pos", "q_slot", "q_kind"):
        got = getattr(step, name).cpu().numpy()
        assert np.array_equal(got[:n_e], getattr(plan, name)), name
    assert np.array_equal(step.cu_q.cpu().numpy(), plan.cu_q)
    assert np.array_equal(step.kv_len.cpu().numpy(), plan.kv_len)
