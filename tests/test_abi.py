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
