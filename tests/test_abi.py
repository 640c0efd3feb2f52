"""CPU-only checks of the C-ABI boundary: the library loads, exports every declared symbol, and the
argument errors that are decided on the host come back as status codes without touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "codecsight.h")
LIB = os.path.join(ROOT, "paper_2604_06036_amd", "libcodecsight.so")


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cs_[a-z_0-9]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.fail(f"{LIB} not built: run `python -m paper_2604_06036_amd.build`")
    return ctypes.CDLL(LIB)


def test_header_declares_the_four_entry_points():
    names = _declared()
    for fn in ("cs_score_compact", "cs_kv_rerotate", "cs_kv_refresh_scatter", "cs_window_prefill_attn"):
        assert fn in names


def test_library_exports_every_declared_symbol(lib):
    for fn in _declared():
        assert hasattr(lib, fn), fn


def test_binding_lists_the_same_symbols():
    from paper_2604_06036_amd import binding
    assert sorted(binding.EXPORTS) == _declared()
    for fn in binding.EXPORTS:
        assert hasattr(binding, fn) or fn == "cs_last_hip_error"


def test_version_and_workspace_queries(lib):
    lib.cs_version.restype = ctypes.c_char_p
    assert b"gfx950" in lib.cs_version()
    lib.cs_score_compact_workspace.restype = ctypes.c_size_t
    lib.cs_score_compact_workspace.argtypes = [ctypes.c_int32] * 5
    assert lib.cs_score_compact_workspace(1, 1, 16, 16, 1) == 16
    assert lib.cs_score_compact_workspace(64, 64, 16, 16, 1) == 17 * 8
    assert lib.cs_score_compact_workspace(65, 65, 16, 16, 1) == 18 * 8


def test_host_side_argument_errors(lib):
    """Null / inconsistent arguments are rejected before any launch (no device is needed)."""
    from paper_2604_06036_amd import binding
    L = binding.lib()
    z = None
    one = ctypes.c_void_p(16)          # a non-null, 16-byte aligned dummy; never dereferenced
    # (a)
    assert L.cs_score_compact(z, z, z, z, z, z, -1, 1, 16, 16, 1, 0, 0, 0, z, z, one, z, 0, z) == binding.CS_EINVAL
    assert L.cs_score_compact(one, z, z, one, one, z, 1, 1, 16, 16, 3, 0, 0, 0, one, one, one, one, 64, z) == binding.CS_EUNSUPPORTED
    assert L.cs_score_compact(one, z, z, one, one, z, 1, 1, 15, 16, 2, 0, 0, 0, one, one, one, one, 64, z) == binding.CS_EINVAL
    assert L.cs_score_compact(one, z, z, one, one, z, 1, 1, 16, 16, 1, 0, 0, 1, one, one, one, one, 64, z) == binding.CS_EINVAL
    assert L.cs_score_compact(z, z, z, one, one, z, 1, 1, 16, 16, 1, 0, 0, 0, one, one, one, one, 64, z) == binding.CS_EINVAL
    assert L.cs_score_compact(one, z, z, one, one, z, 1, 1, 16, 16, 1, 0, 0, 0, one, one, one, z, 0, z) == binding.CS_EWORKSPACE
    assert L.cs_score_compact(one, z, z, one, one, z, 8, 8, 16, 16, 1, 0, 0, 0, one, one, one, one, 8, z) == binding.CS_EWORKSPACE
    # (m) block-to-patch projection
    def proj(**kw):
        a = dict(b=one, cu=one, nf=2, sw=1920, sh=1080, iw=448, ih=448, p=28, gh=16, gw=16, mv=one, it=one)
        a.update(kw)
        return L.cs_project_blocks(a["b"], a["cu"], a["nf"], a["sw"], a["sh"], a["iw"], a["ih"], a["p"], a["gh"],
                                   a["gw"], a["mv"], a["it"], z)
    assert proj(nf=-1) == binding.CS_EINVAL
    assert proj(sw=0) == binding.CS_EINVAL
    assert proj(p=0) == binding.CS_EINVAL
    assert proj(gw=0) == binding.CS_EINVAL
    assert proj(b=z) == binding.CS_EINVAL
    assert proj(mv=z) == binding.CS_EINVAL
    assert proj(it=z) == binding.CS_EINVAL
    assert proj(nf=0, b=z, cu=z, mv=z, it=z) == binding.CS_OK
    assert proj(sw=16385) == binding.CS_EUNSUPPORTED
    assert proj(ih=20000) == binding.CS_EUNSUPPORTED
    assert proj(p=1025) == binding.CS_EUNSUPPORTED
    assert proj(gh=128, gw=57) == binding.CS_EUNSUPPORTED
    assert proj(b=ctypes.c_void_p(24)) == binding.CS_EUNSUPPORTED
    assert proj(mv=ctypes.c_void_p(18)) == binding.CS_EUNSUPPORTED
    # (r) residual proxy
    def resid(**kw):
        a = dict(cur=one, prev=one, f=one, nf=2, sw=1920, sh=1080, pitch=1920, fs=1920 * 1080, cell=4, iw=448,
                 ih=448, p=28, gh=16, gw=16, res=one)
        a.update(kw)
        return L.cs_residual_proxy(a["cur"], a["prev"], a["f"], a["nf"], a["sw"], a["sh"], a["pitch"], a["fs"],
                                   a["cell"], a["iw"], a["ih"], a["p"], a["gh"], a["gw"], a["res"], z)
    assert resid(nf=-1) == binding.CS_EINVAL
    assert resid(sh=0) == binding.CS_EINVAL
    assert resid(pitch=1900) == binding.CS_EINVAL
    assert resid(fs=1920 * 1000) == binding.CS_EINVAL
    assert resid(cur=z) == binding.CS_EINVAL
    assert resid(f=z) == binding.CS_EINVAL
    assert resid(res=z) == binding.CS_EINVAL
    assert resid(nf=0, cur=z, prev=z, f=z, res=z) == binding.CS_OK
    assert resid(cell=5) == binding.CS_EUNSUPPORTED
    assert resid(cell=32) == binding.CS_EUNSUPPORTED
    assert resid(sw=1912, pitch=1912, fs=1912 * 1080) == binding.CS_EUNSUPPORTED      # pitch not a multiple of 16
    assert resid(sw=1910, pitch=1910 + 2, fs=1912 * 1080) == binding.CS_EUNSUPPORTED
    assert resid(fs=1920 * 1080 + 8) == binding.CS_EUNSUPPORTED
    assert resid(prev=ctypes.c_void_p(24)) == binding.CS_EUNSUPPORTED
    assert resid(res=ctypes.c_void_p(18)) == binding.CS_EUNSUPPORTED
    assert resid(sw=64, sh=64, pitch=64, fs=4096, iw=456) == binding.CS_EUNSUPPORTED  # 28*64 < 4*456
    assert resid(sw=20000, pitch=20000, fs=20000 * 1080) == binding.CS_EUNSUPPORTED
    # (p) the device planner
    def plan(**kw):
        a = dict(ot=one, oc=one, nt=one, ko=one, bto=one, mbo=4, btn=one, mbn=4, ns=2, w=8, s=1, nt_=16, t=64,
                 rc=100, qc=100, src=one, dst=one, dl=one, qp=one, qs=one, qk=one, cu=one, kvl=one, oty=one,
                 ocn=one, tot=one, ws=one, wsb=1 << 20)
        a.update(kw)
        return L.cs_plan_refresh(a["ot"], a["oc"], a["nt"], a["ko"], a["bto"], a["mbo"], a["btn"], a["mbn"],
                                 a["ns"], a["w"], a["s"], a["nt_"], a["t"], a["rc"], a["qc"], a["src"], a["dst"],
                                 a["dl"], a["qp"], a["qs"], a["qk"], a["cu"], a["kvl"], a["oty"], a["ocn"],
                                 a["tot"], a["ws"], a["wsb"], z)
    assert plan(ns=-1) == binding.CS_EINVAL
    assert plan(w=0) == binding.CS_EINVAL
    assert plan(s=0) == binding.CS_EINVAL
    assert plan(s=9) == binding.CS_EINVAL
    assert plan(t=0) == binding.CS_EINVAL
    assert plan(nt_=-1) == binding.CS_EINVAL
    assert plan(rc=-1) == binding.CS_EINVAL
    assert plan(mbn=0) == binding.CS_EINVAL
    assert plan(ot=z) == binding.CS_EINVAL
    assert plan(ko=z) == binding.CS_EINVAL
    assert plan(src=z) == binding.CS_EINVAL
    assert plan(qk=z) == binding.CS_EINVAL
    assert plan(tot=z) == binding.CS_EINVAL
    assert plan(cu=z) == binding.CS_EINVAL
    assert plan(rc=1 << 31) == binding.CS_EUNSUPPORTED
    assert plan(ns=1 << 20, w=1 << 11) == binding.CS_EUNSUPPORTED
    assert plan(s=8, t=1 << 28) == binding.CS_EUNSUPPORTED
    need = L.cs_plan_refresh_workspace(2, 8)
    assert need >= 2 * 9 * 16 + 4 * 2 * 4 and need % 256 == 0
    assert L.cs_plan_refresh_workspace(0, 8) == 0 and L.cs_plan_refresh_workspace(2, 0) == 0
    assert plan(ws=z, wsb=0) == binding.CS_EWORKSPACE
    assert plan(wsb=need - 1) == binding.CS_EWORKSPACE
    assert plan(ws=ctypes.c_void_p(24), wsb=need) == binding.CS_EWORKSPACE
    # (b)
    assert L.cs_kv_rerotate(z, z, one, z, one, 4, 1, 1, 64, 0, 64, 64, 1e4, 0, 1, z) == binding.CS_EINVAL
    assert L.cs_kv_rerotate(one, z, one, one, one, 4, 1, 1, 64, 0, 64, 64, 1e4, 0, 1, z) == binding.CS_EINVAL
    assert L.cs_kv_rerotate(one, one, one, z, one, 4, 1, 1, 72, 0, 72, 72, 1e4, 0, 1, z) == binding.CS_EUNSUPPORTED
    assert L.cs_kv_rerotate(one, one, one, z, one, 4, 1, 1, 64, 0, 68, 64, 1e4, 0, 1, z) == binding.CS_EUNSUPPORTED
    assert L.cs_kv_rerotate(one, one, one, z, one, 4, 1, 1, 64, 0, 64, 64, 1e4, 2, 1, z) == binding.CS_EUNSUPPORTED
    assert L.cs_kv_rerotate(one, one, one, z, one, 4, 1, 1, 64, 0, 64, 64, 1e4, 0, 7, z) == binding.CS_EUNSUPPORTED
    assert L.cs_kv_rerotate(one, one, one, z, one, 4, 1, 1, 64, 0, 64, 64, 0.0, 0, 1, z) == binding.CS_EINVAL
    assert L.cs_kv_rerotate(one, one, one, z, one, -1, 1, 1, 64, 0, 64, 64, 1e4, 0, 1, z) == binding.CS_EINVAL
    assert L.cs_kv_rerotate(one, one, one, z, one, 0, 1, 1, 64, 0, 64, 64, 1e4, 0, 1, z) == binding.CS_OK
    # (b') the multi-axis form shares the checks and also needs its axis map
    assert L.cs_kv_rerotate_axes(one, one, one, z, one, z, 4, 1, 1, 64, 0, 64, 64, 1e4, 0, 1, z) == binding.CS_EINVAL
    assert L.cs_kv_rerotate_axes(one, one, one, z, one, one, 4, 1, 1, 72, 0, 72, 72, 1e4, 0, 1, z) == binding.CS_EUNSUPPORTED
    assert L.cs_kv_rerotate_axes(one, one, one, z, one, one, 0, 1, 1, 64, 0, 64, 64, 1e4, 0, 1, z) == binding.CS_OK
    # (c)
    assert L.cs_kv_refresh_scatter(z, one, one, one, one, 4, 1, 64, 64, 64, 1, z) == binding.CS_EINVAL
    assert L.cs_kv_refresh_scatter(one, one, one, one, one, 4, 1, 60, 64, 64, 1, z) == binding.CS_EUNSUPPORTED
    assert L.cs_kv_refresh_scatter(one, one, one, one, one, 0, 1, 64, 64, 64, 1, z) == binding.CS_OK
    # (d)
    def attn(**kw):
        a = dict(q=one, k=one, v=one, cu=one, pos=one, kvl=one, bt=one, maxb=4, bs=16, out=one, nq=8,
                 ns=1, hq=4, hkv=2, d=128, ss=256, sh=128, scale=0.1, dt=1, ws=z, wsb=0, mode=0)
        a.update(kw)
        return L.cs_window_prefill_attn(a["q"], a["k"], a["v"], a["cu"], a["pos"], a["kvl"], a["bt"],
                                        a["maxb"], a["bs"], a["out"], a["nq"], a["ns"], a["hq"], a["hkv"],
                                        a["d"], a["ss"], a["sh"], a["scale"], a["dt"], a["ws"], a["wsb"],
                                        a["mode"], z)
    assert attn(q=z) == binding.CS_EINVAL
    assert attn(hq=5) == binding.CS_EINVAL
    assert attn(d=96) == binding.CS_EUNSUPPORTED
    assert attn(bs=32) == binding.CS_EUNSUPPORTED
    assert attn(hq=34, hkv=2) == binding.CS_EUNSUPPORTED
    assert attn(dt=3) == binding.CS_EUNSUPPORTED
    assert attn(ss=257) == binding.CS_EUNSUPPORTED
    assert attn(nq=0) == binding.CS_OK
    assert attn(nq=-2) == binding.CS_EINVAL
    # bf16 / head_dim 128 keeps its work plan in the workspace: none, too small, unknown plan mode
    need = L.cs_window_prefill_attn_workspace(8, 1, 4, 2, 128, 4, 1)
    assert need > 0
    assert attn() == binding.CS_EWORKSPACE
    assert attn(ws=one, wsb=need - 1) == binding.CS_EWORKSPACE
    assert attn(ws=one, wsb=need, mode=7) == binding.CS_EINVAL
    assert attn(hkv=4, hq=4, ns=1 << 23, ws=one, wsb=1 << 40) == binding.CS_EUNSUPPORTED
    assert attn(scale=0.0) == binding.CS_EINVAL
    assert attn(scale=float("nan")) == binding.CS_EINVAL
    assert attn(scale=-0.1) == binding.CS_EINVAL

    # (c+d) the fused call: its own checks, then those of the two calls
    def fused(**kw):
        a = dict(kn=one, vn=one, slot=one, nt=8, q=one, k=one, v=one, cu=one, pos=one, kvl=one, bt=one, maxb=4, bs=16,
                 out=one, nq=8, ns=1, hq=4, hkv=2, d=128, ss=256, sh=128, scale=0.1, dt=1, ws=z, wsb=0, mode=0)
        a.update(kw)
        return L.cs_refresh_prefill_attn(a["kn"], a["vn"], a["slot"], a["nt"], a["q"], a["k"], a["v"], a["cu"], a["pos"],
                                         a["kvl"], a["bt"], a["maxb"], a["bs"], a["out"], a["nq"], a["ns"], a["hq"],
                                         a["hkv"], a["d"], a["ss"], a["sh"], a["scale"], a["dt"], a["ws"], a["wsb"],
                                         a["mode"], z)
    assert fused(nt=-1) == binding.CS_EINVAL
    assert fused(kn=z) == binding.CS_EINVAL
    assert fused(slot=z) == binding.CS_EINVAL
    assert fused(kn=ctypes.c_void_p(8)) == binding.CS_EUNSUPPORTED          # not 16-byte aligned
    assert fused() == binding.CS_EWORKSPACE                                 # bf16 / 128: the plan needs the workspace
    assert fused(ws=one, wsb=need, mode=7) == binding.CS_EINVAL
    assert fused(scale=0.0, ws=one, wsb=need) == binding.CS_EINVAL
    assert fused(d=96) == binding.CS_EUNSUPPORTED
    assert fused(nq=0, nt=0) == binding.CS_OK

    # the scoring call that allocates nothing serves up to 4,096 streams
    assert L.cs_score_compact_noalloc(one, z, z, one, one, z, 4097, 1, 16, 16, 1, 0, 0, 0, one, one, one, z) == binding.CS_EUNSUPPORTED

    # the measurement aid
    assert L.cs_mfma_rate_probe(z, 1, 1, 0, z) == binding.CS_EINVAL
    assert L.cs_mfma_rate_probe(one, 0, 1, 0, z) == binding.CS_EINVAL
    assert L.cs_mfma_rate_probe(one, 1, 0, 1, z) == binding.CS_EINVAL
    assert L.cs_mfma_rate_probe(one, (1 << 20) + 1, 1, 1, z) == binding.CS_EINVAL


def test_product_package_does_not_import_the_oracle():
    """The HIP path and the oracle share no code: nothing under the package mentions oracle/."""
    pkg = os.path.join(ROOT, "paper_2604_06036_amd")
    for dirpath, _, files in os.walk(pkg):
        for name in files:
            if name.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, name)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, flags=re.M), name
    for name in os.listdir(os.path.join(ROOT, "oracle")):
        if name.endswith(".py"):
            text = open(os.path.join(ROOT, "oracle", name)).read()
            assert "paper_2604_06036_amd" not in text, name
