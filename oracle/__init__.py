"""ctypes front end of the CPU oracle (test infrastructure only).

Only tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this package.  The product package never does, and this package never
imports the product package.

All arrays are numpy, host memory.  BF16 tensors are ``uint16`` bit patterns.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_LIB = None

INT8, MXFP4 = 0, 1
PER_TOKEN, PER_CHANNEL = 0, 1


def lib():
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        _LIB = C.CDLL(path)
    return _LIB


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


def num_threads():
    f = lib().msd_oracle_num_threads
    f.restype = C.c_int
    return int(f())


def decompose_int8(x_bf16, fractional=False):
    """Sec. 3.2 two-pass INT8 decomposition of every row of x (uint16 BF16 bits, [M][K]).
    Returns q1, q2 (int8 [M][K]), alpha, beta (float32 [M])."""
    x = _c(x_bf16, np.uint16)
    M, K = x.shape
    q1 = np.empty((M, K), np.int8)
    q2 = np.empty((M, K), np.int8)
    al = np.empty(M, np.float32)
    be = np.empty(M, np.float32)
    lib().msd_oracle_decompose_int8(_p(x), C.c_int64(M), C.c_int64(K), C.c_int64(K),
                                    C.c_int(int(fractional)), _p(q1), _p(q2), _p(al), _p(be))
    return q1, q2, al, be


def gemm_w8a16(x_bf16, W, w_scale, fractional=False, out_bf16=False, taps=False):
    """Alg. 1.  Returns y ([M][N] float32, or uint16 BF16 bits) and, with taps=True, a dict
    with q1, q2, alpha, beta, acc1, acc2, overflow."""
    x = _c(x_bf16, np.uint16)
    W = _c(W, np.int8)
    s = _c(w_scale, np.float32)
    M, K = x.shape
    N = W.shape[0]
    assert W.shape[1] == K and s.shape == (N,)
    y = np.empty((M, N), np.uint16 if out_bf16 else np.float32)
    t = {}
    if taps:
        t = dict(q1=np.empty((M, K), np.int8), q2=np.empty((M, K), np.int8),
                 alpha=np.empty(M, np.float32), beta=np.empty(M, np.float32),
                 acc1=np.empty((M, N), np.int32), acc2=np.empty((M, N), np.int32))
    ovf = C.c_int(0)
    lib().msd_oracle_gemm_w8a16(_p(x), C.c_int64(M), C.c_int64(K), C.c_int64(K), _p(W), _p(s),
                                C.c_int64(N), C.c_int(int(fractional)), _p(y),
                                C.c_int(int(out_bf16)), C.c_int64(N), _p(t.get("q1")),
                                _p(t.get("q2")), _p(t.get("alpha")), _p(t.get("beta")),
                                _p(t.get("acc1")), _p(t.get("acc2")), C.byref(ovf))
    if taps:
        t["overflow"] = bool(ovf.value)
        return y, t
    return y


def moe_gemm_w8a16(x_bf16, expert_offsets, W, w_scale, out_bf16=False):
    """Grouped form of Alg. 1 for mixture-of-experts layers (Sec. 7.5: the decomposition is per activation
    row, so the grouped GEMM is Alg. 1 applied per expert).  x_bf16 [T][K] sorted by expert, expert e owns
    rows [expert_offsets[e], expert_offsets[e+1]); W [E][N][K], w_scale [E][N].  Rows past expert_offsets[E]
    are returned as zeros."""
    offs = np.asarray(expert_offsets, np.int64)
    E, N, K = W.shape
    T = x_bf16.shape[0]
    assert offs.shape == (E + 1,) and offs[0] == 0 and np.all(np.diff(offs) >= 0) and offs[-1] <= T
    y = np.zeros((T, N), np.uint16 if out_bf16 else np.float32)
    for e in range(E):
        r0, r1 = int(offs[e]), int(offs[e + 1])
        if r1 > r0:
            y[r0:r1] = gemm_w8a16(x_bf16[r0:r1], W[e], w_scale[e], out_bf16=out_bf16)
    return y


def truth_gemm_w8(x_bf16, W, w_scale):
    x = _c(x_bf16, np.uint16)
    W = _c(W, np.int8)
    s = _c(w_scale, np.float32)
    M, K = x.shape
    N = W.shape[0]
    y = np.empty((M, N), np.float64)
    lib().msd_oracle_truth_gemm_w8(_p(x), C.c_int64(M), C.c_int64(K), C.c_int64(K), _p(W), _p(s),
                                   C.c_int64(N), _p(y))
    return y


def dequant_gemm_w8a16(x_bf16, W, w_scale):
    x = _c(x_bf16, np.uint16)
    W = _c(W, np.int8)
    s = _c(w_scale, np.float32)
    M, K = x.shape
    N = W.shape[0]
    y = np.empty((M, N), np.float32)
    lib().msd_oracle_dequant_gemm_w8a16(_p(x), C.c_int64(M), C.c_int64(K), C.c_int64(K), _p(W),
                                        _p(s), C.c_int64(N), _p(y))
    return y


def decompose_mxfp4(x_bf16, variant=3):
    """Alg. 2.  Returns q1, q2 (uint8 nibble-packed [M][K/2], low nibble = even k) and the
    E8M0 byte of alpha ([M][K/32]); beta's byte is alpha's minus 4 (minus 3 for variant 1).
    variant 4: the E2M1-grid ablation (codes are OCP E2M1 nibbles, beta's byte is alpha's minus 2)."""
    x = _c(x_bf16, np.uint16)
    M, K = x.shape
    assert K % 32 == 0
    q1 = np.empty((M, K // 2), np.uint8)
    q2 = np.empty((M, K // 2), np.uint8)
    e = np.empty((M, K // 32), np.uint8)
    lib().msd_oracle_decompose_mxfp4(_p(x), C.c_int64(M), C.c_int64(K), C.c_int64(K),
                                     C.c_int(variant), _p(q1), _p(q2), _p(e))
    return q1, q2, e


def gemm_w4a16(x_bf16, W_fp4, W_e8m0, variant=3, out_bf16=False, taps=False):
    x = _c(x_bf16, np.uint16)
    Wq = _c(W_fp4, np.uint8)
    We = _c(W_e8m0, np.uint8)
    M, K = x.shape
    N = Wq.shape[0]
    assert Wq.shape == (N, K // 2) and We.shape == (N, K // 32)
    y = np.empty((M, N), np.uint16 if out_bf16 else np.float32)
    t = {}
    if taps:
        t = dict(q1=np.empty((M, K // 2), np.uint8), q2=np.empty((M, K // 2), np.uint8),
                 e8m0=np.empty((M, K // 32), np.uint8))
    lib().msd_oracle_gemm_w4a16(_p(x), C.c_int64(M), C.c_int64(K), C.c_int64(K), _p(Wq), _p(We),
                                C.c_int64(N), C.c_int(variant), _p(y), C.c_int(int(out_bf16)),
                                C.c_int64(N), _p(t.get("q1")), _p(t.get("q2")), _p(t.get("e8m0")))
    return (y, t) if taps else y


def moe_gemm_w4a16(x_bf16, expert_offsets, W_fp4, W_e8m0, out_bf16=False):
    """Grouped form of the W4A16 GEMM (Sec. 7.5; Alg. 2 + Sec. 3.4.1 per expert).  W_fp4 [E][N][K/2],
    W_e8m0 [E][N][K/32]; rows past expert_offsets[E] are returned as zeros."""
    offs = np.asarray(expert_offsets, np.int64)
    E, N = W_fp4.shape[:2]
    T = x_bf16.shape[0]
    assert offs.shape == (E + 1,) and offs[0] == 0 and np.all(np.diff(offs) >= 0) and offs[-1] <= T
    y = np.zeros((T, N), np.uint16 if out_bf16 else np.float32)
    for e in range(E):
        r0, r1 = int(offs[e]), int(offs[e + 1])
        if r1 > r0:
            y[r0:r1] = gemm_w4a16(x_bf16[r0:r1], W_fp4[e], W_e8m0[e], out_bf16=out_bf16)
    return y


def truth_gemm_w4(x_bf16, W_fp4, W_e8m0):
    x = _c(x_bf16, np.uint16)
    Wq = _c(W_fp4, np.uint8)
    We = _c(W_e8m0, np.uint8)
    M, K = x.shape
    N = Wq.shape[0]
    y = np.empty((M, N), np.float64)
    lib().msd_oracle_truth_gemm_w4(_p(x), C.c_int64(M), C.c_int64(K), C.c_int64(K), _p(Wq),
                                   _p(We), C.c_int64(N), _p(y))
    return y


def _attn_args(q_bf16, Kc, Vc, k_scale, v_scale, kv_len):
    q = _c(q_bf16, np.uint16)
    Kc = _c(Kc, np.int8)
    Vc = _c(Vc, np.int8)
    ks = _c(k_scale, np.float32)
    vs = _c(v_scale, np.float32)
    B, Hq, d = q.shape
    _, Hkv, L, _ = Kc.shape
    assert Kc.shape == (B, Hkv, L, d) and Vc.shape == Kc.shape and Hq % Hkv == 0
    kl = None if kv_len is None else _c(kv_len, np.int32)
    return q, Kc, Vc, ks, vs, kl, B, Hq, Hkv, d, L


def attn_decode(q_bf16, Kc, Vc, k_scale, v_scale, scale_mode, kv_len=None, taps=False, lowprec=False):
    """Alg. 3 (untiled).  Returns out float32 [B][Hq][d] (+ taps dict).  lowprec: the low-precision arithmetic
    of Sec. 4.4 ("optimisation opportunities"): integer S merge, FP16 decomposition of P."""
    q, Kc, Vc, ks, vs, kl, B, Hq, Hkv, d, L = _attn_args(q_bf16, Kc, Vc, k_scale, v_scale, kv_len)
    if scale_mode == PER_TOKEN:
        assert ks.shape == (B, Hkv, L) and vs.shape == (B, Hkv, L)
    else:
        assert ks.shape == (Hkv, d) and vs.shape == (Hkv, d)
    out = np.empty((B, Hq, d), np.float32)
    t = {}
    if taps:
        t = dict(q1=np.empty((B, Hq, d), np.int8), q2=np.empty((B, Hq, d), np.int8),
                 alpha_q=np.empty((B, Hq), np.float32), s1=np.zeros((B, Hq, L), np.int32),
                 s2=np.zeros((B, Hq, L), np.int32), p=np.zeros((B, Hq, L), np.float32),
                 p1=np.zeros((B, Hq, L), np.int8), p2=np.zeros((B, Hq, L), np.int8))
    fn = lib().msd_oracle_attn_decode_lowprec if lowprec else lib().msd_oracle_attn_decode
    fn(_p(q), _p(Kc), _p(Vc), _p(ks), _p(vs), C.c_int(scale_mode),
                                 C.c_int(B), C.c_int(Hq), C.c_int(Hkv), C.c_int(d), _p(kl),
                                 C.c_int64(L), _p(out), _p(t.get("q1")), _p(t.get("q2")),
                                 _p(t.get("alpha_q")), _p(t.get("s1")), _p(t.get("s2")),
                                 _p(t.get("p")), _p(t.get("p1")), _p(t.get("p2")))
    return (out, t) if taps else out


def truth_attn(q_bf16, Kc, Vc, k_scale, v_scale, scale_mode, kv_len=None):
    q, Kc, Vc, ks, vs, kl, B, Hq, Hkv, d, L = _attn_args(q_bf16, Kc, Vc, k_scale, v_scale, kv_len)
    out = np.empty((B, Hq, d), np.float64)
    lib().msd_oracle_truth_attn(_p(q), _p(Kc), _p(Vc), _p(ks), _p(vs), C.c_int(scale_mode),
                                C.c_int(B), C.c_int(Hq), C.c_int(Hkv), C.c_int(d), _p(kl),
                                C.c_int64(L), _p(out))
    return out


def mla_decode(q_bf16, C_lat, scale, scale_mode, dv, sm_scale, kv_len=None, taps=False):
    """Alg. 3 over a latent KV cache (Sec. 4.4, Sec. 7.3): q [B][Hq][dk] BF16 bits, C_lat [B][L][dk] int8 (keys =
    whole rows, values = their first dv channels, one shared row per token for all heads), scale [B][L]
    (per token) or [dk] (per channel), score scale sm_scale.  Returns out float32 [B][Hq][dv] (+ taps)."""
    q = _c(q_bf16, np.uint16)
    Cl = _c(C_lat, np.int8)
    sc = _c(scale, np.float32)
    B, Hq, dk = q.shape
    _, L, ld = Cl.shape
    assert Cl.shape[0] == B and ld >= dk and 0 < dv <= dk
    assert sc.shape == ((B, L) if scale_mode == PER_TOKEN else (dk,))
    kl = None if kv_len is None else _c(kv_len, np.int32)
    out = np.empty((B, Hq, dv), np.float32)
    t = {}
    if taps:
        t = dict(q1=np.empty((B, Hq, dk), np.int8), q2=np.empty((B, Hq, dk), np.int8),
                 alpha_q=np.empty((B, Hq), np.float32), s1=np.zeros((B, Hq, L), np.int32),
                 s2=np.zeros((B, Hq, L), np.int32))
    lib().msd_oracle_mla_decode(_p(q), _p(Cl), C.c_int64(ld), _p(sc), C.c_int(scale_mode), C.c_int(B), C.c_int(Hq),
                                C.c_int(dk), C.c_int(dv), C.c_double(sm_scale), _p(kl), C.c_int64(L), _p(out),
                                _p(t.get("q1")), _p(t.get("q2")), _p(t.get("alpha_q")), _p(t.get("s1")),
                                _p(t.get("s2")))
    return (out, t) if taps else out


def truth_mla(q_bf16, C_lat, scale, scale_mode, dv, sm_scale, kv_len=None):
    q = _c(q_bf16, np.uint16)
    Cl = _c(C_lat, np.int8)
    sc = _c(scale, np.float32)
    B, Hq, dk = q.shape
    _, L, ld = Cl.shape
    kl = None if kv_len is None else _c(kv_len, np.int32)
    out = np.empty((B, Hq, dv), np.float64)
    lib().msd_oracle_truth_mla(_p(q), _p(Cl), C.c_int64(ld), _p(sc), C.c_int(scale_mode), C.c_int(B), C.c_int(Hq),
                               C.c_int(dk), C.c_int(dv), C.c_double(sm_scale), _p(kl), C.c_int64(L), _p(out))
    return out
