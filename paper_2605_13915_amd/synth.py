"""Seeded synthetic inputs shaped like the paper's workloads (numpy, host memory).

This module serves both the CPU oracle's tests and the HIP path's tests / benchmark.
It holds none of the method's arithmetic: it only draws random tensors and performs the
offline preparation that happens before the method runs (BF16 storage of activations,
offline weight quantisation, KV-cache quantisation).  It imports neither the oracle
nor the HIP binding.

Workload recipe (Sec. 6.1 "Data generation" uses random INT8 weights with per-channel
scales and random activations; the decode regime b << m, n of Sec. 3.8; the GQA decode
shape of Sec. 4.4.1):
  activations  fp32 N(0,1); for the outlier configs 1 % of the K channels (seeded choice)
               are multiplied by 50 in every row; stored as BF16 (round-to-nearest-even)
  INT8 weights integers uniform in [-127, 127]; s_W ~ U(0.001, 0.01) fp32 per output channel
  MXFP4 weights fp32 N(0, std 0.02) quantised offline to OCP MXFP4: per 32 along K,
               shared exponent floor(log2(max|w|)) - 2, elements RNE to E2M1, saturating at 6
  KV cache     fp32 N(0,1) rows of d, scale = rowmax/127 per token and head, codes RNE
"""
import numpy as np

BASE_SEED = 20260513


def seed_for(cfg: int, shape_index: int = 0) -> int:
    return BASE_SEED + 1000 * cfg + shape_index


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> BF16 bit patterns (uint16), round-to-nearest-even; finite inputs."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(h, np.uint16).astype(np.uint32) << 16).view(np.float32)


def activations(seed: int, M: int, K: int, outliers: bool = True, dist: str = "normal",
                scale: float = 1.0) -> np.ndarray:
    """BF16 bit patterns [M][K]."""
    rng = np.random.default_rng(seed)
    if dist == "normal":
        x = rng.standard_normal((M, K), dtype=np.float32)
    elif dist == "uniform":
        x = rng.uniform(-1.0, 1.0, (M, K)).astype(np.float32)
    elif dist == "laplace":
        x = rng.laplace(0.0, 1.0, (M, K)).astype(np.float32)
    else:
        raise ValueError(dist)
    x *= np.float32(scale)
    if outliers:
        n_out = int(round(0.01 * K))
        idx = rng.permutation(K)[:n_out]
        x[:, idx] *= np.float32(50.0)
    return f32_to_bf16_bits(x)


def int8_weights(seed: int, N: int, K: int):
    """W int8 [N][K] uniform in [-127,127]; s_W float32 [N] ~ U(0.001, 0.01)."""
    rng = np.random.default_rng(seed + 500)
    W = rng.integers(-127, 128, size=(N, K), dtype=np.int8)
    s = rng.uniform(0.001, 0.01, N).astype(np.float32)
    return W, s


_E2M1_MAG = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], np.float32)


def quantize_mxfp4(w: np.ndarray):
    """Offline OCP MXFP4 quantisation of fp32 w [N][K] along K in blocks of 32.
    Returns nibble-packed codes uint8 [N][K/2] (low nibble = even k; bit 3 sign, bits 2..0
    E2M1 magnitude index) and E8M0 bytes uint8 [N][K/32] (value 2^(byte-127))."""
    N, K = w.shape
    assert K % 32 == 0
    wb = w.reshape(N, K // 32, 32).astype(np.float32)
    amax = np.abs(wb).max(axis=2)
    with np.errstate(divide="ignore"):
        e = np.where(amax > 0, np.floor(np.log2(np.maximum(amax, np.float32(1e-38)))), -125.0)
    e = e.astype(np.int32) - 2               # E2M1's largest binade is 2^2
    e = np.clip(e, -127, 127)
    scaled = wb / np.exp2(e.astype(np.float32))[:, :, None]
    mag = np.minimum(np.abs(scaled), np.float32(6.0))
    # nearest E2M1 magnitude, ties to the even mantissa (index parity even)
    dist = np.abs(mag[..., None] - _E2M1_MAG[None, None, None, :])
    best = dist.min(axis=-1, keepdims=True)
    cand = dist == best
    even_first = np.where(cand & (np.arange(8) % 2 == 0), 0, np.where(cand, 1, 2))
    idx = even_first.argmin(axis=-1).astype(np.uint8)
    sign = (scaled < 0) & (idx > 0)
    nib = (idx | (sign.astype(np.uint8) << 3)).reshape(N, K)
    packed = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)
    return packed, (e + 127).astype(np.uint8)


def mxfp4_weights(seed: int, N: int, K: int, std: float = 0.02, chunk: int = 2048):
    rng = np.random.default_rng(seed + 700)
    codes = np.empty((N, K // 2), np.uint8)
    exps = np.empty((N, K // 32), np.uint8)
    for n0 in range(0, N, chunk):
        n1 = min(N, n0 + chunk)
        w = rng.standard_normal((n1 - n0, K), dtype=np.float32) * np.float32(std)
        codes[n0:n1], exps[n0:n1] = quantize_mxfp4(w)
    return codes, exps


def dequantize_mxfp4(codes: np.ndarray, exps: np.ndarray) -> np.ndarray:
    """Decode OCP MXFP4 (for tests of this module and of the fp64 truth)."""
    N, K2 = codes.shape
    nib = np.empty((N, K2 * 2), np.uint8)
    nib[:, 0::2] = codes & 15
    nib[:, 1::2] = codes >> 4
    v = _E2M1_MAG[nib & 7] * np.where(nib & 8, np.float32(-1), np.float32(1))
    return (v.reshape(N, -1, 32) * np.exp2(exps.astype(np.float32) - 127)[:, :, None]).reshape(N, -1)


def kv_cache_per_token(seed: int, B: int, Hkv: int, L: int, d: int, chunk_tokens: int = 1 << 16):
    """INT8 K, V [B][Hkv][L][d] with per-token-per-head fp32 scales [B][Hkv][L]."""
    rng = np.random.default_rng(seed + 900)
    out = []
    for _ in range(2):
        codes = np.empty((B * Hkv * L, d), np.int8)
        scales = np.empty(B * Hkv * L, np.float32)
        for t0 in range(0, B * Hkv * L, chunk_tokens):
            t1 = min(B * Hkv * L, t0 + chunk_tokens)
            x = rng.standard_normal((t1 - t0, d), dtype=np.float32)
            s = np.abs(x).max(axis=1) / np.float32(127.0)
            s = np.maximum(s, np.float32(1e-30))
            codes[t0:t1] = np.clip(np.rint(x / s[:, None]), -127, 127).astype(np.int8)
            scales[t0:t1] = s
        out.append((codes.reshape(B, Hkv, L, d), scales.reshape(B, Hkv, L)))
    (Kc, ks), (Vc, vs) = out
    return Kc, ks, Vc, vs


def kv_cache_per_channel(seed: int, B: int, Hkv: int, L: int, d: int):
    """INT8 K, V [B][Hkv][L][d] with per-channel fp32 scales [Hkv][d] (the paper's layout)."""
    rng = np.random.default_rng(seed + 950)
    out = []
    for _ in range(2):
        x = rng.standard_normal((B, Hkv, L, d), dtype=np.float32)
        s = np.abs(x).max(axis=(0, 2)) / np.float32(127.0)
        codes = np.clip(np.rint(x / s[None, :, None, :]), -127, 127).astype(np.int8)
        out.append((codes, s.astype(np.float32)))
    (Kc, ks), (Vc, vs) = out
    return Kc, ks, Vc, vs


def queries(seed: int, B: int, Hq: int, d: int) -> np.ndarray:
    rng = np.random.default_rng(seed + 990)
    return f32_to_bf16_bits(rng.standard_normal((B, Hq, d), dtype=np.float32))
