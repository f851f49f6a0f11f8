"""The C-ABI library loads and exports every function include/msd.h declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "msd.h")
LIB = os.path.join(ROOT, "paper_2605_13915_amd", "libmsd.so")


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(msd_[a-z0-9_]+)\s*\(", src)))


def test_header_declares_the_four_entry_points():
    names = declared_functions()
    for must in ("msd_decompose", "msd_gemm_w8a16", "msd_gemm_w4a16", "msd_attn_decode_int8kv"):
        assert must in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        import __graft_entry__
        __graft_entry__.build()
    lib = ctypes.CDLL(LIB)
    for name in declared_functions():
        assert hasattr(lib, name), name
    lib.msd_version.restype = ctypes.c_char_p
    assert lib.msd_version().decode().count(".") == 1


def test_workspace_queries_and_host_side_validation():
    # size queries and argument validation run on the host: no device is touched
    lib = ctypes.CDLL(LIB)
    i64 = ctypes.c_int64
    lib.msd_gemm_w8a16_workspace_bytes.restype = ctypes.c_size_t
    lib.msd_gemm_w8a16_workspace_bytes.argtypes = [i64, i64, i64]
    small = lib.msd_gemm_w8a16_workspace_bytes(1, 4096, 4096)
    big = lib.msd_gemm_w8a16_workspace_bytes(128, 4096, 4096)
    assert small >= 2 * 4096 + 4 and big > small
    lib.msd_decompose.argtypes = [ctypes.c_int, ctypes.c_void_p, i64, i64, i64, ctypes.c_void_p,
                                  ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    assert lib.msd_decompose(7, None, 1, 16, 16, None, None, None, None) == -1      # bad fmt
    assert lib.msd_decompose(0, None, 1, 16, 8, None, None, None, None) == -2       # ldx < K
    assert lib.msd_decompose(0, None, 1, 16, 16, None, None, None, None) == -1      # null pointers
    assert lib.msd_decompose(0, None, 0, 16, 16, None, None, None, None) == 0       # empty: no-op
    assert lib.msd_decompose(1, ctypes.c_void_p(256), 1, 48, 48, ctypes.c_void_p(256), ctypes.c_void_p(256),
                             ctypes.c_void_p(256), None) == -2                      # K % 32 != 0
    lib.msd_stream_read.argtypes = [ctypes.c_void_p, i64, i64, ctypes.c_void_p]
    assert lib.msd_stream_read(ctypes.c_void_p(256), 16, 100, None) == -2            # row_bytes % 256 != 0
    assert lib.msd_stream_read(None, 16, 256, None) == -1                           # null pointer
    assert lib.msd_stream_read(None, 0, 256, None) == 0                             # empty: no-op
