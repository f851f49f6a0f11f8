"""Thin Python binding over the C-ABI library (argument marshalling only).

PyTorch provides device memory and the stream; every step of the path runs inside
``libmsd.so``.  The functions carry the names of the C entry points declared in
``include/msd.h``.  There is no fallback: if the library is missing, loading raises.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmsd.so")

MSD_INT8, MSD_MXFP4 = 0, 1
MSD_F32, MSD_BF16 = 0, 1
MSD_PER_TOKEN, MSD_PER_CHANNEL = 0, 1
MSD_VARIANT_MAIN, MSD_VARIANT_INT8_FRACTIONAL, MSD_VARIANT_MXFP4_V1, MSD_VARIANT_MXFP4_V2 = 0, 1, 2, 3
MSD_VARIANT_MXFP4_E2M1 = 4
MSD_VARIANT_ATTN_LOWPREC = 5

_ERR = {-1: "MSD_ERR_INVALID_ARG", -2: "MSD_ERR_SHAPE", -3: "MSD_ERR_WORKSPACE", -4: "MSD_ERR_HIP",
        -5: "MSD_ERR_UNSUPPORTED", -6: "MSD_ERR_STATIC_SCRATCH"}


class MsdError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (where, _ERR.get(code, "?"), code))


class Taps(C.Structure):
    _fields_ = [("q1", C.c_void_p), ("q2", C.c_void_p), ("scale", C.c_void_p),
                ("acc1", C.c_void_p), ("acc2", C.c_void_p), ("p1", C.c_void_p), ("p2", C.c_void_p)]


_lib = None


def lib():
    """Load libmsd.so (built by paper_2605_13915_amd/build.py); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("HIP library %s is missing: run `python -m paper_2605_13915_amd.build` "
                               "(or __graft_entry__.build()) first" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        i64, vp, ci, sz = C.c_int64, C.c_void_p, C.c_int, C.c_size_t
        L.msd_last_hip_error.restype = ci
        L.msd_version.restype = C.c_char_p
        L.msd_decompose.argtypes = [ci, vp, i64, i64, i64, vp, vp, vp, vp]
        L.msd_decompose_variant.argtypes = [ci] + L.msd_decompose.argtypes
        gemm8 = [vp, i64, i64, i64, vp, vp, i64, vp, ci, i64, vp, sz, vp, vp]
        gemm4 = [vp, i64, i64, i64, vp, vp, i64, vp, ci, i64, vp, sz, vp, vp]
        L.msd_gemm_w8a16.argtypes = gemm8
        L.msd_gemm_w8a16_packed.argtypes = gemm8
        L.msd_gemm_w8a16_packed.restype = ci
        L.msd_packed_weights_w8_bytes.argtypes = [i64, i64]
        L.msd_packed_weights_w8_bytes.restype = sz
        L.msd_pack_weights_w8.argtypes = [vp, i64, i64, vp, vp]
        L.msd_pack_weights_w8.restype = ci
        L.msd_gemm_w8a16_static.argtypes = [vp, i64, i64, i64, vp, vp, i64, vp, ci, i64, vp]
        L.msd_gemm_w8a16_static.restype = ci
        L.msd_gemm_w8a16_static_scratch_bytes.argtypes = []
        L.msd_gemm_w8a16_static_scratch_bytes.restype = sz
        L.msd_dequant_gemm_w8a16.argtypes = gemm8
        L.msd_probe_mfma_w8a16.argtypes = gemm8
        L.msd_gemm_w4a16.argtypes = gemm4
        L.msd_gemm_w4a16_packed.argtypes = gemm4
        L.msd_gemm_w4a16_packed.restype = ci
        L.msd_packed_weights_w4_bytes.argtypes = [i64, i64]
        L.msd_packed_weights_w4_bytes.restype = sz
        L.msd_packed_scales_w4_bytes.argtypes = [i64, i64]
        L.msd_packed_scales_w4_bytes.restype = sz
        L.msd_pack_weights_w4.argtypes = [vp, vp, i64, i64, vp, vp, vp]
        L.msd_pack_weights_w4.restype = ci
        L.msd_dequant_gemm_w4a16.argtypes = gemm4
        L.msd_probe_mfma_w4a16.argtypes = gemm4
        L.msd_gemm_w8a16_variant.argtypes = [ci] + gemm8
        L.msd_gemm_w4a16_variant.argtypes = [ci] + gemm4
        for f in (L.msd_gemm_w8a16_workspace_bytes, L.msd_gemm_w4a16_workspace_bytes,
                  L.msd_dequant_gemm_workspace_bytes):
            f.argtypes = [i64, i64, i64]
            f.restype = sz
        L.msd_attn_decode_int8kv.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, i64, vp, ci, vp, sz,
                                             vp, vp]
        L.msd_mla_decode_int8kv.argtypes = [vp, vp, i64, vp, ci, ci, ci, ci, ci, C.c_float, vp, i64, vp, ci, vp, sz,
                                            vp, vp]
        L.msd_dequant_mla_decode_int8kv.argtypes = L.msd_mla_decode_int8kv.argtypes
        L.msd_mla_decode_int8kv_workspace_bytes.argtypes = [ci, ci, i64]
        L.msd_mla_decode_int8kv_workspace_bytes.restype = sz
        L.msd_moe_gemm_w8a16.argtypes = [vp, i64, i64, i64, vp, ci, vp, vp, i64, vp, ci, i64, vp, sz, vp]
        L.msd_moe_gemm_w4a16.argtypes = L.msd_moe_gemm_w8a16.argtypes
        L.msd_dequant_attn_decode_int8kv.argtypes = L.msd_attn_decode_int8kv.argtypes
        L.msd_attn_decode_int8kv_variant.argtypes = [ci] + L.msd_attn_decode_int8kv.argtypes
        L.msd_attn_decode_int8kv_variant.restype = ci
        L.msd_attn_decode_int8kv_workspace_bytes.argtypes = [ci, ci, ci, ci, i64]
        L.msd_attn_decode_int8kv_workspace_bytes.restype = sz
        L.msd_stream_read.argtypes = [vp, i64, i64, vp]
        L.msd_stream_read_linear.argtypes = [vp, i64, vp]
        L.msd_probe_mfma_rate.argtypes = [ci, vp, ci, vp]
        L.msd_probe_mfma_rate.restype = ci
        L.msd_stream_read_linear.restype = ci
        L.msd_probe_lds_fill_rate.argtypes = [vp, i64, i64, ci, ci, vp]
        L.msd_probe_lds_fill_rate.restype = ci
        for name in ("msd_decompose", "msd_gemm_w8a16", "msd_gemm_w4a16", "msd_attn_decode_int8kv",
                     "msd_dequant_gemm_w8a16", "msd_dequant_gemm_w4a16", "msd_stream_read", "msd_probe_mfma_w8a16",
                     "msd_probe_mfma_w4a16", "msd_decompose_variant", "msd_gemm_w8a16_variant",
                     "msd_gemm_w4a16_variant", "msd_dequant_attn_decode_int8kv", "msd_moe_gemm_w8a16",
                     "msd_moe_gemm_w4a16", "msd_mla_decode_int8kv", "msd_dequant_mla_decode_int8kv"):
            getattr(L, name).restype = ci
        _lib = L
    return _lib


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc, where):
    if rc != 0:
        raise MsdError(rc, where)


def _dev(t, dtype, name):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype):
        raise TypeError("%s must be a CUDA tensor of dtype %s" % (name, dtype))
    return t


_ws_cache = {}


def workspace(nbytes, device):
    """A cached uint8 device buffer of at least nbytes (torch allocations are 256-B aligned)."""
    key = (str(device),)
    buf = _ws_cache.get(key)
    if buf is None or buf.numel() < nbytes:
        buf = torch.empty(max(int(nbytes), 1 << 20), dtype=torch.uint8, device=device)
        _ws_cache[key] = buf
    return buf


def _out_code(dtype):
    if dtype == torch.float32:
        return MSD_F32
    if dtype == torch.bfloat16:
        return MSD_BF16
    raise TypeError("out dtype must be float32 or bfloat16")


class Prepared:
    """One C-ABI call with every argument marshalled once.  ``prepared()`` enqueues it again on the
    stream it was prepared for (a few hundred nanoseconds of Python instead of ~10 us), which is what
    tight loops and HIP-graph capture want.  Holds references to the tensors it points into."""

    __slots__ = ("fn", "args", "keep", "name", "out")

    def __init__(self, fn, args, keep, name, out):
        self.fn, self.args, self.keep, self.name, self.out = fn, args, keep, name, out

    def __call__(self):
        rc = self.fn(*self.args)
        if rc != 0:
            raise MsdError(rc, self.name)
        return self.out


def msd_decompose(fmt, x):
    """x: bf16 [M][K] (row stride may exceed K).  Returns (q1, q2, scale) device tensors."""
    return msd_decompose_variant(None, fmt, x)


def msd_decompose_variant(variant, fmt, x):
    """msd_decompose with the decomposition constants of `variant` (None: the entry point without one)."""
    _dev(x, torch.bfloat16, "x")
    M, K = x.shape
    assert x.stride(1) == 1
    if fmt == MSD_INT8:
        q1 = torch.empty((M, K), dtype=torch.int8, device=x.device)
        q2 = torch.empty_like(q1)
        sc = torch.empty((M,), dtype=torch.float32, device=x.device)
    else:
        q1 = torch.empty((M, K // 2), dtype=torch.uint8, device=x.device)
        q2 = torch.empty_like(q1)
        sc = torch.empty((M, K // 32), dtype=torch.uint8, device=x.device)
    args = (fmt, _ptr(x), M, K, x.stride(0) if M > 1 else max(K, x.stride(0)), _ptr(q1), _ptr(q2), _ptr(sc),
            _stream())
    if variant is None:
        _check(lib().msd_decompose(*args), "msd_decompose")
    else:
        _check(lib().msd_decompose_variant(variant, *args), "msd_decompose_variant")
    return q1, q2, sc


def _gemm_common(fn_name, ws_fn, x, w_args, N, out_dtype, taps, y, ws, prepare=False, lead=()):
    L = lib()
    M, K = x.shape
    if y is None:
        y = torch.empty((M, N), dtype=out_dtype, device=x.device)
    if ws is None:
        ws = workspace(getattr(L, ws_fn)(M, K, N), x.device)
    tp = None
    keep = {}
    if taps:
        if "w8a16" in fn_name:
            keep = dict(q1=torch.empty((M, K), dtype=torch.int8, device=x.device),
                        q2=torch.empty((M, K), dtype=torch.int8, device=x.device),
                        scale=torch.empty((M,), dtype=torch.float32, device=x.device),
                        acc1=torch.empty((M, N), dtype=torch.int32, device=x.device),
                        acc2=torch.empty((M, N), dtype=torch.int32, device=x.device))
        else:
            keep = dict(q1=torch.empty((M, K // 2), dtype=torch.uint8, device=x.device),
                        q2=torch.empty((M, K // 2), dtype=torch.uint8, device=x.device),
                        scale=torch.empty((M, K // 32), dtype=torch.uint8, device=x.device))
        tp = Taps(keep["q1"].data_ptr(), keep["q2"].data_ptr(), keep["scale"].data_ptr(),
                  keep["acc1"].data_ptr() if "acc1" in keep else None,
                  keep["acc2"].data_ptr() if "acc2" in keep else None)
    ldx = x.stride(0) if M > 1 else max(K, x.stride(0))
    args = (*lead, _ptr(x), M, K, ldx, *w_args, N, _ptr(y), _out_code(y.dtype), y.stride(0), _ptr(ws), ws.numel(),
            C.byref(tp) if tp is not None else None, _stream())
    if prepare:
        return Prepared(getattr(L, fn_name), args, (x, y, ws, keep, tp), fn_name, y)
    rc = getattr(L, fn_name)(*args)
    _check(rc, fn_name)
    return (y, keep) if taps else y


def msd_gemm_w8a16(x, W, w_scale, out_dtype=torch.float32, taps=False, y=None, ws=None, prepare=False):
    _dev(x, torch.bfloat16, "x"); _dev(W, torch.int8, "W"); _dev(w_scale, torch.float32, "w_scale")
    assert W.is_contiguous() and W.shape[1] == x.shape[1] and w_scale.shape[0] == W.shape[0]
    return _gemm_common("msd_gemm_w8a16", "msd_gemm_w8a16_workspace_bytes", x, (_ptr(W), _ptr(w_scale)),
                        W.shape[0], out_dtype, taps, y, ws, prepare)


def msd_pack_weights_w8(W):
    """W int8 [N][K] (K % 64 == 0) -> the packed array msd_gemm_w8a16_packed reads (one-time, offline)."""
    _dev(W, torch.int8, "W")
    assert W.is_contiguous()
    N, K = W.shape
    packed = torch.empty(lib().msd_packed_weights_w8_bytes(N, K), dtype=torch.int8, device=W.device)
    _check(lib().msd_pack_weights_w8(_ptr(W), N, K, _ptr(packed), _stream()), "msd_pack_weights_w8")
    return packed


def msd_gemm_w8a16_packed(x, W_packed, w_scale, out_dtype=torch.float32, taps=False, y=None, ws=None, prepare=False):
    """msd_gemm_w8a16 on weights packed by msd_pack_weights_w8; N is taken from w_scale."""
    _dev(x, torch.bfloat16, "x"); _dev(W_packed, torch.int8, "W_packed"); _dev(w_scale, torch.float32, "w_scale")
    N, K = w_scale.shape[0], x.shape[1]
    assert W_packed.numel() == lib().msd_packed_weights_w8_bytes(N, K)
    return _gemm_common("msd_gemm_w8a16_packed", "msd_gemm_w8a16_workspace_bytes", x, (_ptr(W_packed), _ptr(w_scale)),
                        N, out_dtype, taps, y, ws, prepare)


def msd_gemm_w8a16_static(x, W, w_scale, y, prepare=False):
    """msd_gemm_w8a16 on the library's built-in scratch buffer; y is the caller's (nothing is allocated)."""
    _dev(x, torch.bfloat16, "x"); _dev(W, torch.int8, "W"); _dev(w_scale, torch.float32, "w_scale")
    assert W.is_contiguous() and W.shape[1] == x.shape[1] and w_scale.shape[0] == W.shape[0]
    assert isinstance(y, torch.Tensor) and y.is_cuda and y.shape == (x.shape[0], W.shape[0])
    M, K = x.shape
    ldx = x.stride(0) if M > 1 else max(K, x.stride(0))
    args = (_ptr(x), M, K, ldx, _ptr(W), _ptr(w_scale), W.shape[0], _ptr(y), _out_code(y.dtype), y.stride(0),
            _stream())
    fn = lib().msd_gemm_w8a16_static
    if prepare:
        return Prepared(fn, args, (x, W, w_scale, y), "msd_gemm_w8a16_static", y)
    _check(fn(*args), "msd_gemm_w8a16_static")
    return y


def msd_gemm_w8a16_variant(variant, x, W, w_scale, out_dtype=torch.float32, taps=False, y=None, ws=None,
                           prepare=False):
    _dev(x, torch.bfloat16, "x"); _dev(W, torch.int8, "W"); _dev(w_scale, torch.float32, "w_scale")
    assert W.is_contiguous() and W.shape[1] == x.shape[1] and w_scale.shape[0] == W.shape[0]
    return _gemm_common("msd_gemm_w8a16_variant", "msd_gemm_w8a16_workspace_bytes", x, (_ptr(W), _ptr(w_scale)),
                        W.shape[0], out_dtype, taps, y, ws, prepare, lead=(int(variant),))


def msd_dequant_gemm_w8a16(x, W, w_scale, out_dtype=torch.float32, y=None, ws=None, prepare=False):
    _dev(x, torch.bfloat16, "x"); _dev(W, torch.int8, "W"); _dev(w_scale, torch.float32, "w_scale")
    assert W.is_contiguous()
    return _gemm_common("msd_dequant_gemm_w8a16", "msd_dequant_gemm_workspace_bytes", x,
                        (_ptr(W), _ptr(w_scale)), W.shape[0], out_dtype, False, y, ws, prepare)


def msd_probe_mfma_w8a16(x, W, w_scale, y=None, ws=None, prepare=False):
    """Measurement aid: the many-row W8A16 kernel's MFMA sequence without its data movement (y is meaningless)."""
    _dev(x, torch.bfloat16, "x"); _dev(W, torch.int8, "W"); _dev(w_scale, torch.float32, "w_scale")
    assert W.is_contiguous() and W.shape[1] == x.shape[1]
    return _gemm_common("msd_probe_mfma_w8a16", "msd_gemm_w8a16_workspace_bytes", x, (_ptr(W), _ptr(w_scale)),
                        W.shape[0], torch.float32, False, y, ws, prepare)


def msd_probe_mfma_w4a16(x, W_fp4, W_e8m0, y=None, ws=None, prepare=False):
    """Measurement aid: the many-row W4A16 kernel's MFMA sequence without its data movement (y is meaningless)."""
    _dev(x, torch.bfloat16, "x"); _dev(W_fp4, torch.uint8, "W_fp4"); _dev(W_e8m0, torch.uint8, "W_e8m0")
    return _gemm_common("msd_probe_mfma_w4a16", "msd_gemm_w4a16_workspace_bytes", x, (_ptr(W_fp4), _ptr(W_e8m0)),
                        W_fp4.shape[0], torch.float32, False, y, ws, prepare)


def msd_gemm_w4a16(x, W_fp4, W_e8m0, out_dtype=torch.float32, taps=False, y=None, ws=None, prepare=False):
    _dev(x, torch.bfloat16, "x"); _dev(W_fp4, torch.uint8, "W_fp4"); _dev(W_e8m0, torch.uint8, "W_e8m0")
    assert W_fp4.is_contiguous() and W_e8m0.is_contiguous() and W_fp4.shape[1] * 2 == x.shape[1]
    return _gemm_common("msd_gemm_w4a16", "msd_gemm_w4a16_workspace_bytes", x, (_ptr(W_fp4), _ptr(W_e8m0)),
                        W_fp4.shape[0], out_dtype, taps, y, ws, prepare)


def msd_pack_weights_w4(W_fp4, W_e8m0):
    """W_fp4 uint8 [N][K/2], W_e8m0 uint8 [N][K/32] (K % 512 == 0) -> (packed_fp4, packed_e8m0), the arrays
    msd_gemm_w4a16_packed reads (one-time, offline)."""
    _dev(W_fp4, torch.uint8, "W_fp4"); _dev(W_e8m0, torch.uint8, "W_e8m0")
    assert W_fp4.is_contiguous() and W_e8m0.is_contiguous()
    N, K = W_fp4.shape[0], W_fp4.shape[1] * 2
    Wp = torch.empty(lib().msd_packed_weights_w4_bytes(N, K), dtype=torch.uint8, device=W_fp4.device)
    Ep = torch.empty(lib().msd_packed_scales_w4_bytes(N, K), dtype=torch.uint8, device=W_fp4.device)
    _check(lib().msd_pack_weights_w4(_ptr(W_fp4), _ptr(W_e8m0), N, K, _ptr(Wp), _ptr(Ep), _stream()),
           "msd_pack_weights_w4")
    return Wp, Ep


def msd_gemm_w4a16_packed(x, packed_fp4, packed_e8m0, N, out_dtype=torch.float32, taps=False, y=None, ws=None,
                          prepare=False):
    """msd_gemm_w4a16 on the arrays of msd_pack_weights_w4; N (output channels) cannot be read off them."""
    _dev(x, torch.bfloat16, "x"); _dev(packed_fp4, torch.uint8, "packed_fp4"); _dev(packed_e8m0, torch.uint8, "packed_e8m0")
    K = x.shape[1]
    assert packed_fp4.numel() == lib().msd_packed_weights_w4_bytes(N, K)
    assert packed_e8m0.numel() == lib().msd_packed_scales_w4_bytes(N, K)
    return _gemm_common("msd_gemm_w4a16_packed", "msd_gemm_w4a16_workspace_bytes", x, (_ptr(packed_fp4), _ptr(packed_e8m0)),
                        N, out_dtype, taps, y, ws, prepare)


def msd_gemm_w4a16_variant(variant, x, W_fp4, W_e8m0, out_dtype=torch.float32, taps=False, y=None, ws=None,
                           prepare=False):
    _dev(x, torch.bfloat16, "x"); _dev(W_fp4, torch.uint8, "W_fp4"); _dev(W_e8m0, torch.uint8, "W_e8m0")
    assert W_fp4.is_contiguous() and W_e8m0.is_contiguous() and W_fp4.shape[1] * 2 == x.shape[1]
    return _gemm_common("msd_gemm_w4a16_variant", "msd_gemm_w4a16_workspace_bytes", x,
                        (_ptr(W_fp4), _ptr(W_e8m0)), W_fp4.shape[0], out_dtype, taps, y, ws, prepare,
                        lead=(int(variant),))


def msd_dequant_gemm_w4a16(x, W_fp4, W_e8m0, out_dtype=torch.float32, y=None, ws=None, prepare=False):
    _dev(x, torch.bfloat16, "x"); _dev(W_fp4, torch.uint8, "W_fp4"); _dev(W_e8m0, torch.uint8, "W_e8m0")
    return _gemm_common("msd_dequant_gemm_w4a16", "msd_dequant_gemm_workspace_bytes", x,
                        (_ptr(W_fp4), _ptr(W_e8m0)), W_fp4.shape[0], out_dtype, False, y, ws, prepare)


def msd_moe_gemm_w8a16(x, expert_offsets, W, w_scale, out_dtype=torch.float32, y=None, ws=None, prepare=False):
    """x: bf16 [T][K], rows sorted by expert; expert_offsets: int32 device tensor [E+1]; W: int8 [E][N][K];
    w_scale: float [E][N].  Returns y [T][N]."""
    _dev(x, torch.bfloat16, "x"); _dev(W, torch.int8, "W"); _dev(w_scale, torch.float32, "w_scale")
    _dev(expert_offsets, torch.int32, "expert_offsets")
    T, K = x.shape
    E, N, K2 = W.shape
    assert K2 == K and W.is_contiguous() and w_scale.shape == (E, N) and w_scale.is_contiguous()
    assert expert_offsets.numel() == E + 1 and expert_offsets.is_contiguous()
    L = lib()
    if y is None:
        y = torch.empty((T, N), dtype=out_dtype, device=x.device)
    if ws is None:
        ws = workspace(L.msd_gemm_w8a16_workspace_bytes(T, K, N), x.device)
    ldx = x.stride(0) if T > 1 else max(K, x.stride(0))
    args = (_ptr(x), T, K, ldx, _ptr(expert_offsets), E, _ptr(W), _ptr(w_scale), N, _ptr(y), _out_code(y.dtype),
            y.stride(0), _ptr(ws), ws.numel(), _stream())
    if prepare:
        return Prepared(L.msd_moe_gemm_w8a16, args, (x, expert_offsets, W, w_scale, y, ws), "msd_moe_gemm_w8a16", y)
    _check(L.msd_moe_gemm_w8a16(*args), "msd_moe_gemm_w8a16")
    return y


def msd_moe_gemm_w4a16(x, expert_offsets, W_fp4, W_e8m0, out_dtype=torch.float32, y=None, ws=None, prepare=False):
    """x: bf16 [T][K], rows sorted by expert; expert_offsets: int32 device tensor [E+1]; W_fp4: uint8 [E][N][K/2];
    W_e8m0: uint8 [E][N][K/32].  Returns y [T][N]."""
    _dev(x, torch.bfloat16, "x"); _dev(W_fp4, torch.uint8, "W_fp4"); _dev(W_e8m0, torch.uint8, "W_e8m0")
    _dev(expert_offsets, torch.int32, "expert_offsets")
    T, K = x.shape
    E, N, K2 = W_fp4.shape
    assert K2 * 2 == K and W_fp4.is_contiguous() and W_e8m0.shape == (E, N, K // 32) and W_e8m0.is_contiguous()
    assert expert_offsets.numel() == E + 1 and expert_offsets.is_contiguous()
    L = lib()
    if y is None:
        y = torch.empty((T, N), dtype=out_dtype, device=x.device)
    if ws is None:
        ws = workspace(L.msd_gemm_w4a16_workspace_bytes(T, K, N), x.device)
    ldx = x.stride(0) if T > 1 else max(K, x.stride(0))
    args = (_ptr(x), T, K, ldx, _ptr(expert_offsets), E, _ptr(W_fp4), _ptr(W_e8m0), N, _ptr(y), _out_code(y.dtype),
            y.stride(0), _ptr(ws), ws.numel(), _stream())
    if prepare:
        return Prepared(L.msd_moe_gemm_w4a16, args, (x, expert_offsets, W_fp4, W_e8m0, y, ws), "msd_moe_gemm_w4a16", y)
    _check(L.msd_moe_gemm_w4a16(*args), "msd_moe_gemm_w4a16")
    return y


def msd_stream_read(t, prepare=False):
    """Measurement aid: bare read of the 2-D byte tensor t (rows of a multiple of 256 bytes)."""
    assert t.is_cuda and t.dim() == 2 and t.is_contiguous() and t.element_size() == 1
    args = (_ptr(t), t.shape[0], t.shape[1], _stream())
    call = Prepared(lib().msd_stream_read, args, (t,), "msd_stream_read", None)
    return call if prepare else call()


def msd_probe_mfma_rate(fmt, operands, iters):
    """Measurement aid: 2048 waves x 8 * iters matrix instructions on the operand bits in the 64 KB tensor `operands`;
    returns the number of scalar operations issued (2 per multiply-add)."""
    assert operands.is_cuda and operands.is_contiguous() and operands.numel() * operands.element_size() >= 65536
    _check(lib().msd_probe_mfma_rate(int(fmt), _ptr(operands), int(iters), _stream()), "msd_probe_mfma_rate")
    return 2048 * 8 * int(iters) * 2 * (65536 if fmt == MSD_MXFP4 else 32768)


def msd_probe_lds_fill_rate(t, hot_bytes, hot_parts, rounds):
    """Measurement aid: 256 workgroups x `rounds` x 32 KB of asynchronous LDS fills out of the byte tensor t, of
    which hot_parts quarters come from the shared window t[:hot_bytes]; returns the bytes moved."""
    assert t.is_cuda and t.is_contiguous() and t.element_size() == 1
    _check(lib().msd_probe_lds_fill_rate(_ptr(t), t.numel(), int(hot_bytes), int(hot_parts), int(rounds), _stream()),
           "msd_probe_lds_fill_rate")
    return 256 * int(rounds) * 32768


def msd_stream_read_linear(t, prepare=False):
    """Measurement aid: bare linear read of the contiguous byte tensor t (a multiple of 16 bytes)."""
    assert t.is_cuda and t.is_contiguous() and t.element_size() == 1
    args = (_ptr(t), t.numel(), _stream())
    call = Prepared(lib().msd_stream_read_linear, args, (t,), "msd_stream_read_linear", None)
    return call if prepare else call()


def msd_attn_decode_int8kv(q, K, V, k_scale, v_scale, scale_mode, kv_len=None, out_dtype=torch.float32,
                           taps=False, out=None, ws=None, prepare=False, _fn="msd_attn_decode_int8kv", variant=None):
    _dev(q, torch.bfloat16, "q"); _dev(K, torch.int8, "K"); _dev(V, torch.int8, "V")
    _dev(k_scale, torch.float32, "k_scale"); _dev(v_scale, torch.float32, "v_scale")
    B, Hq, d = q.shape
    _, Hkv, Lmax, _ = K.shape
    assert q.is_contiguous() and K.is_contiguous() and V.is_contiguous()
    L = lib()
    if out is None:
        out = torch.empty((B, Hq, d), dtype=out_dtype, device=q.device)
    if ws is None:
        ws = workspace(L.msd_attn_decode_int8kv_workspace_bytes(B, Hq, Hkv, d, Lmax), q.device)
    tp = None
    keep = {}
    if taps:
        keep = dict(q1=torch.empty((B, Hq, d), dtype=torch.int8, device=q.device),
                    q2=torch.empty((B, Hq, d), dtype=torch.int8, device=q.device),
                    scale=torch.empty((B, Hq), dtype=torch.float32, device=q.device),
                    acc1=torch.zeros((B, Hq, Lmax), dtype=torch.int32, device=q.device),
                    acc2=torch.zeros((B, Hq, Lmax), dtype=torch.int32, device=q.device),
                    p1=torch.zeros((B, Hq, Lmax), dtype=torch.int8, device=q.device),
                    p2=torch.zeros((B, Hq, Lmax), dtype=torch.int8, device=q.device))
        tp = Taps(*(keep[k].data_ptr() for k in ("q1", "q2", "scale", "acc1", "acc2", "p1", "p2")))
    if kv_len is not None:
        _dev(kv_len, torch.int32, "kv_len")
    args = (_ptr(q), _ptr(K), _ptr(V), _ptr(k_scale), _ptr(v_scale), scale_mode, B, Hq, Hkv, d, _ptr(kv_len),
            Lmax, _ptr(out), _out_code(out.dtype), _ptr(ws), ws.numel(),
            C.byref(tp) if tp is not None else None, _stream())
    if variant is not None:
        _fn, args = "msd_attn_decode_int8kv_variant", (int(variant),) + args
    if prepare:
        return Prepared(getattr(L, _fn), args, (q, K, V, k_scale, v_scale, kv_len, out, ws, keep, tp), _fn, out)
    rc = getattr(L, _fn)(*args)
    _check(rc, _fn)
    return (out, keep) if taps else out


def msd_attn_decode_int8kv_variant(variant, q, K, V, k_scale, v_scale, scale_mode, **kw):
    """msd_attn_decode_int8kv with the arithmetic of `variant` (MSD_VARIANT_ATTN_LOWPREC)."""
    return msd_attn_decode_int8kv(q, K, V, k_scale, v_scale, scale_mode, variant=variant, **kw)


def msd_dequant_attn_decode_int8kv(q, K, V, k_scale, v_scale, scale_mode, kv_len=None, out_dtype=torch.float32,
                                   out=None, ws=None, prepare=False):
    """Comparison kernel: K and V lifted to BF16 in registers, BF16 matrix instructions."""
    return msd_attn_decode_int8kv(q, K, V, k_scale, v_scale, scale_mode, kv_len, out_dtype, False, out, ws, prepare,
                                  _fn="msd_dequant_attn_decode_int8kv")


def msd_mla_decode_int8kv(q, C_lat, scale, scale_mode, sm_scale, kv_len=None, out_dtype=torch.float32, taps=False,
                          out=None, ws=None, prepare=False):
    """q: bf16 [B][Hq][576]; C_lat: int8 [B][L][ld] (keys = first 576 channels of a row, values = first 512);
    scale: float [B][L] (per token) or [576] (per channel).  Returns out [B][Hq][512] (+ taps)."""
    _dev(q, torch.bfloat16, "q"); _dev(C_lat, torch.int8, "C_lat"); _dev(scale, torch.float32, "scale")
    B, Hq, dk = q.shape
    _, Lmax, ld = C_lat.shape
    assert q.is_contiguous() and C_lat.is_contiguous() and scale.is_contiguous()
    L = lib()
    dv = 512
    if out is None:
        out = torch.empty((B, Hq, dv), dtype=out_dtype, device=q.device)
    if ws is None:
        ws = workspace(L.msd_mla_decode_int8kv_workspace_bytes(B, Hq, Lmax), q.device)
    tp = None
    keep = {}
    if taps:
        keep = dict(q1=torch.empty((B, Hq, dk), dtype=torch.int8, device=q.device),
                    q2=torch.empty((B, Hq, dk), dtype=torch.int8, device=q.device),
                    scale=torch.empty((B, Hq), dtype=torch.float32, device=q.device),
                    acc1=torch.zeros((B, Hq, Lmax), dtype=torch.int32, device=q.device),
                    acc2=torch.zeros((B, Hq, Lmax), dtype=torch.int32, device=q.device))
        tp = Taps(*(keep[k].data_ptr() for k in ("q1", "q2", "scale", "acc1", "acc2")))
    if kv_len is not None:
        _dev(kv_len, torch.int32, "kv_len")
    args = (_ptr(q), _ptr(C_lat), ld, _ptr(scale), scale_mode, B, Hq, dk, dv, float(sm_scale), _ptr(kv_len), Lmax,
            _ptr(out), _out_code(out.dtype), _ptr(ws), ws.numel(), C.byref(tp) if tp is not None else None, _stream())
    if prepare:
        return Prepared(L.msd_mla_decode_int8kv, args, (q, C_lat, scale, kv_len, out, ws, keep, tp),
                        "msd_mla_decode_int8kv", out)
    _check(L.msd_mla_decode_int8kv(*args), "msd_mla_decode_int8kv")
    return (out, keep) if taps else out


def msd_dequant_mla_decode_int8kv(q, C_lat, scale, scale_mode, sm_scale, kv_len=None, out_dtype=torch.float32,
                                  out=None, ws=None, prepare=False):
    """The dequantise-then-BF16 comparison kernel on the arguments of msd_mla_decode_int8kv (no taps)."""
    _dev(q, torch.bfloat16, "q"); _dev(C_lat, torch.int8, "C_lat"); _dev(scale, torch.float32, "scale")
    B, Hq, dk = q.shape
    _, Lmax, ld = C_lat.shape
    assert q.is_contiguous() and C_lat.is_contiguous() and scale.is_contiguous()
    L = lib()
    if out is None:
        out = torch.empty((B, Hq, 512), dtype=out_dtype, device=q.device)
    if ws is None:
        ws = workspace(L.msd_mla_decode_int8kv_workspace_bytes(B, Hq, Lmax), q.device)
    if kv_len is not None:
        _dev(kv_len, torch.int32, "kv_len")
    args = (_ptr(q), _ptr(C_lat), ld, _ptr(scale), scale_mode, B, Hq, dk, 512, float(sm_scale), _ptr(kv_len), Lmax,
            _ptr(out), _out_code(out.dtype), _ptr(ws), ws.numel(), None, _stream())
    if prepare:
        return Prepared(L.msd_dequant_mla_decode_int8kv, args, (q, C_lat, scale, kv_len, out, ws),
                        "msd_dequant_mla_decode_int8kv", out)
    _check(L.msd_dequant_mla_decode_int8kv(*args), "msd_dequant_mla_decode_int8kv")
    return out
