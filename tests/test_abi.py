"""The C-ABI library loads without a GPU and exports every symbol include/fxp.h declares;
argument errors are reported before anything touches a device."""
import ctypes
import os
import re

from paper_2207_08822_amd import build as fxp_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def load():
    path = fxp_build.LIB if os.path.exists(fxp_build.LIB) else fxp_build.build()
    return ctypes.CDLL(path)


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "fxp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fxp_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    L = load()
    names = declared_symbols()
    assert {"fxp_scale", "fxp_map", "fxp_gemm", "fxp_unmap", "fxp_linear_fwd", "fxp_linear_bwd", "fxp_gemm_unmap",
            "fxp_scale_map", "fxp_unmap_i8", "fxp_workspace_bytes", "fxp_strerror", "fxp_version"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_host_only_entry_points_and_argument_errors():
    L = load()
    L.fxp_strerror.restype = ctypes.c_char_p
    assert L.fxp_strerror(0) == b"ok"
    assert L.fxp_version() >= 100
    L.fxp_workspace_bytes.restype = ctypes.c_size_t
    L.fxp_workspace_bytes.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64]
    assert L.fxp_workspace_bytes(0, 1 << 20, 0, 0) >= 4096
    assert L.fxp_workspace_bytes(1, 100, 200, 300) >= 100 * 300 + 200 * 300
    assert L.fxp_workspace_bytes(99, 1, 1, 1) == 0
    vp, i64, u64, ci, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64, ctypes.c_int, ctypes.c_size_t
    L.fxp_map.argtypes = [vp, i64, i64, vp, vp, vp, u64, u64, ci, ci, vp]
    # these return before any launch: NULL pointers, bad sizes, bad modes
    assert L.fxp_map(None, 4, 4, None, None, None, 0, 0, 0, 8, None) == -1
    assert L.fxp_map(None, -1, 4, None, None, None, 0, 0, 0, 8, None) == -2
    fake = ctypes.c_void_p(4096)
    assert L.fxp_map(fake, 4, 4, fake, fake, None, 0, 0, 7, 8, None) == -5
    assert L.fxp_map(fake, 4, 4, fake, fake, None, 0, 0, 0, 9, None) == -6
    L.fxp_gemm.argtypes = [ci, ci, i64, i64, i64, vp, i64, vp, i64, vp, i64, vp, sz, vp]
    assert L.fxp_gemm(0, 1, 4, 4, 200000, fake, 200000, fake, 200000, fake, 4, None, 0, None) == -8
    assert L.fxp_gemm(0, 1, 4, 4, 16, fake, 8, fake, 16, fake, 4, None, 0, None) == -2
    assert L.fxp_gemm(0, 0, 4, 4, 16, fake, 16, fake, 16, fake, 4, None, 0, None) == -4    # needs workspace
    L.fxp_scale.argtypes = [vp, sz, vp, vp, sz, vp]
    assert L.fxp_scale(fake, 16, fake, None, 0, None) == -4
