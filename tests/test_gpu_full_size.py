"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py times
(the entry points without observation points, caller-provided output and workspace; the GEMMs on the canonical
weight arrays against the oracle and, bit for bit against that result, on the packed arrays bench.py times by
default).

cfg1 (W8A16 decode) and the small W4 / attention shapes are compared element by element in full; so are the
latent-cache and grouped-GEMM shapes of the bench legs (sampled batch entries; every routed row).  For the
shapes whose oracle run would take minutes (cfg2 prefill, W4 with 4096 rows, attention at L = 32768) the
oracle computes a sample of complete activation rows, resp. complete batch entries -- rows and batch entries
are independent, so the sampled results are exact full-size results -- spread over first, last and interior
tiles.  To keep input generation to seconds, the MXFP4 weight matrix and the long KV cache are a seeded
slab repeated along N resp. L (every tile and split of the kernels is still exercised; the values a tile
sees do not matter to the bar).  Bars as everywhere: 1e-6 (W8), 2e-6 (W4), 1e-3 (attention) relative L2."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_13915_amd import synth
from gpu_util import bf16_to_dev, to_dev, rel_l2

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def msd():
    from paper_2605_13915_amd import binding
    binding.lib()
    return binding


def _rows(M, n=10, seed=0):
    """first, last, tile-boundary and random interior rows"""
    fixed = [0, 1, 127, 128, 255, 256, M // 2, M - 129, M - 2, M - 1]
    rng = np.random.default_rng(seed)
    rows = sorted(set([r for r in fixed if 0 <= r < M] + list(rng.integers(0, M, n))))
    return np.array(rows)


def _rows_every_tile(M, tile, seed=0):
    """the rows of _rows plus one random row out of every `tile` consecutive rows: every row tile of the
    kernel's schedule is looked at"""
    rng = np.random.default_rng(seed + 1)
    per_tile = [t * tile + int(rng.integers(0, min(tile, M - t * tile))) for t in range((M + tile - 1) // tile)]
    return np.array(sorted(set(list(_rows(M, 4, seed)) + per_tile)))


@pytest.mark.parametrize("N", [4096, 14336])
def test_cfg1_w8a16_decode_full(msd, N):
    K = 4096
    W, s = synth.int8_weights(synth.seed_for(1, 10 + N), N, K)
    Wd, sd = to_dev(W), to_dev(s)
    Wp = msd.msd_pack_weights_w8(Wd)
    for M in (1, 8, 32, 128):
        x = synth.activations(synth.seed_for(1, M), M, K, outliers=True)
        ref = oracle.gemm_w8a16(x, W, s)
        y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        msd.msd_gemm_w8a16(bf16_to_dev(x), Wd, sd, y=y)
        torch.cuda.synchronize()
        yh = y.cpu().numpy()
        assert np.all(np.isfinite(yh))
        assert rel_l2(yh, ref) <= 1e-6
        for m in range(M):
            assert rel_l2(yh[m], ref[m]) <= 1e-6
        yp = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        msd.msd_gemm_w8a16_packed(bf16_to_dev(x), Wp, sd, y=yp)
        torch.cuda.synchronize()
        assert torch.equal(y, yp)


@pytest.fixture(scope="module")
def prefill_inputs():
    K = 8192
    x = synth.activations(synth.seed_for(2, 0), 8192, K, outliers=True)
    W, s = synth.int8_weights(synth.seed_for(2, 1), 28672, K)
    return x, W, s


@pytest.mark.parametrize("M,N", [(2048, 8192), (8192, 8192), (2048, 28672), (8192, 28672)])
def test_cfg2_w8a16_prefill_sampled_rows(msd, prefill_inputs, M, N):
    x, W, s = prefill_inputs
    x, W, s = x[:M], W[:N], s[:N]
    y = torch.empty((M, N), dtype=torch.float32, device="cuda")
    xd, Wd, sd = bf16_to_dev(x), to_dev(W), to_dev(s)
    msd.msd_gemm_w8a16(xd, Wd, sd, y=y)
    torch.cuda.synchronize()
    rows = _rows_every_tile(M, 128, seed=M + N)   # the kernel's row tile is 128 activation rows
    assert bool(torch.isfinite(y).all())         # every element, not only the sampled rows
    Wp = msd.msd_pack_weights_w8(Wd)
    del Wd
    yp = torch.empty((M, N), dtype=torch.float32, device="cuda")
    msd.msd_gemm_w8a16_packed(xd, Wp, sd, y=yp)
    torch.cuda.synchronize()
    assert torch.equal(y, yp)
    del yp, Wp
    yh = y[torch.from_numpy(rows).cuda()].cpu().numpy()
    del y
    torch.cuda.empty_cache()
    ref = oracle.gemm_w8a16(x[rows], W, s)
    assert np.all(np.isfinite(yh))
    for i in range(len(rows)):
        assert rel_l2(yh[i], ref[i]) <= 1e-6, rows[i]


@pytest.fixture(scope="module")
def w4_weights():
    K, N, slab = 8192, 28672, 2048
    codes, exps = synth.mxfp4_weights(synth.seed_for(3, 0), slab, K)
    return np.tile(codes, (N // slab, 1)), np.tile(exps, (N // slab, 1))


@pytest.mark.parametrize("M", [1, 32, 4096])
def test_cfg3_w4a16(msd, w4_weights, M):
    codes, exps = w4_weights
    K, N = 8192, codes.shape[0]
    x = synth.activations(synth.seed_for(3, M), M, K, outliers=True)
    y = torch.empty((M, N), dtype=torch.float32, device="cuda")
    xd, cd, ed = bf16_to_dev(x), to_dev(codes), to_dev(exps)
    msd.msd_gemm_w4a16(xd, cd, ed, y=y)
    torch.cuda.synchronize()
    rows = np.arange(M) if M <= 32 else _rows_every_tile(M, 128, seed=M)   # 128-row tiles: 32 + boundary rows
    assert bool(torch.isfinite(y).all())
    Wp, Ep = msd.msd_pack_weights_w4(cd, ed)
    yp = torch.empty((M, N), dtype=torch.float32, device="cuda")
    msd.msd_gemm_w4a16_packed(xd, Wp, Ep, N, y=yp)
    torch.cuda.synchronize()
    assert torch.equal(y, yp)
    del yp, Wp, Ep
    yh = y[torch.from_numpy(rows).cuda()].cpu().numpy()
    ref = oracle.gemm_w4a16(x[rows], codes, exps)
    assert np.all(np.isfinite(yh))
    for i in range(len(rows)):
        assert rel_l2(yh[i], ref[i]) <= 2e-6, rows[i]


@pytest.mark.parametrize("L,mode", [(4096, "token"), (4096, "channel"), (32768, "token")])
def test_cfg4_attention(msd, L, mode):
    B, Hq, Hkv, d, slab = 16, 32, 8, 128, 4096
    q = synth.queries(synth.seed_for(4, L), B, Hq, d)
    if mode == "token":
        Kc, ks, Vc, vs = synth.kv_cache_per_token(synth.seed_for(4, 1), B, Hkv, slab, d)
        rep = L // slab
        Kc, Vc = np.tile(Kc, (1, 1, rep, 1)), np.tile(Vc, (1, 1, rep, 1))
        ks, vs = np.tile(ks, (1, 1, rep)), np.tile(vs, (1, 1, rep))
        omode, gmode = oracle.PER_TOKEN, msd.MSD_PER_TOKEN
    else:
        Kc, ks, Vc, vs = synth.kv_cache_per_channel(synth.seed_for(4, 2), B, Hkv, L, d)
        omode, gmode = oracle.PER_CHANNEL, msd.MSD_PER_CHANNEL
    out = msd.msd_attn_decode_int8kv(bf16_to_dev(q), to_dev(Kc), to_dev(Vc), to_dev(ks), to_dev(vs), gmode)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    sel = list(range(B)) if L <= 4096 else [0, 9, 15]
    if mode == "token":
        ref = oracle.attn_decode(q[sel], Kc[sel], Vc[sel], ks[sel], vs[sel], omode)
    else:
        ref = oracle.attn_decode(q[sel], Kc[sel], Vc[sel], ks, vs, omode)
    assert np.all(np.isfinite(o))
    for i, b in enumerate(sel):
        for h in range(Hq):
            assert rel_l2(o[b, h], ref[i, h]) <= 1e-3, (b, h)


@pytest.mark.parametrize("Hq,L", [(16, 4096), (128, 4096), (16, 32768)])
def test_latent_cache_attention_bench_shapes(msd, Hq, L):
    """The three shapes of bench.py's latent-cache leg (B = 32, per-token scales): every output row of a sample
    of batch entries (all of them are independent) against the oracle."""
    B, slab = 32, 4096
    q = synth.queries(synth.seed_for(9, Hq + L), B, Hq, 576)
    Cl, sc, _, _ = synth.kv_cache_per_token(synth.seed_for(9, 3), B, 1, slab, 576)
    Cl, sc = np.ascontiguousarray(Cl[:, 0]), np.ascontiguousarray(sc[:, 0])
    rep = L // slab
    Cl, sc = np.tile(Cl, (1, rep, 1)), np.tile(sc, (1, rep))
    sm = 1.0 / np.sqrt(192.0)
    out = msd.msd_mla_decode_int8kv(bf16_to_dev(q), to_dev(Cl), to_dev(sc), msd.MSD_PER_TOKEN, sm)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert np.all(np.isfinite(o))
    sel = [0, 13, 31]
    ref = oracle.mla_decode(q[sel], Cl[sel], sc[sel], oracle.PER_TOKEN, 512, sm)
    for i, b in enumerate(sel):
        for h in range(Hq):
            assert rel_l2(o[b, h], ref[i, h]) <= 1e-3, (b, h)


@pytest.mark.parametrize("T", [16, 256])
def test_grouped_gemm_bench_shapes(msd, T):
    """The grouped (mixture-of-experts) GEMMs at the sizes of bench.py's leg: 64 INT8 experts and 128 MXFP4
    experts of N = 2048, K = 4096, multinomial routing.  The experts are one seeded matrix with a sign per
    expert (enough to tell them apart; the bytes a kernel sees do not matter to the bar); every routed row is
    compared with the oracle's product of that row with its expert."""
    N, K = 2048, 4096
    rng = np.random.default_rng(91 + T)
    x = synth.activations(synth.seed_for(8, T), T, K, outliers=True)
    xd = bf16_to_dev(x)
    # W8A16
    E = 64
    W0, s0 = synth.int8_weights(synth.seed_for(8, 1), N, K)
    sign = np.where(rng.integers(0, 2, E) == 1, 1, -1).astype(np.int8)
    W = W0[None] * sign[:, None, None]
    s = np.repeat(s0[None], E, 0) * (1.0 + np.arange(E, dtype=np.float32)[:, None] / E)
    counts = rng.multinomial(T, np.ones(E) / E)
    offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    y = torch.full((T, N), float("nan"), dtype=torch.float32, device="cuda")
    msd.msd_moe_gemm_w8a16(xd, to_dev(offs), to_dev(W), to_dev(s), y=y)
    torch.cuda.synchronize()
    yh = y.cpu().numpy()
    for e in range(E):
        r0, r1 = int(offs[e]), int(offs[e + 1])
        if r1 > r0:
            ref = oracle.gemm_w8a16(x[r0:r1], W[e], s[e])
            assert rel_l2(yh[r0:r1], ref) <= 1e-6, e
    del W, y
    # W4A16
    E = 128
    codes0, exps0 = synth.mxfp4_weights(synth.seed_for(8, 2), N, K)
    flip = (rng.integers(0, 2, E) == 1)
    codes = np.where(flip[:, None, None], codes0[None] ^ np.uint8(0x88), codes0[None])
    exps = np.repeat(exps0[None], E, 0)
    counts = rng.multinomial(T, np.ones(E) / E)
    offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    y = torch.full((T, N), float("nan"), dtype=torch.float32, device="cuda")
    msd.msd_moe_gemm_w4a16(xd, to_dev(offs), to_dev(codes), to_dev(exps), y=y)
    torch.cuda.synchronize()
    yh = y.cpu().numpy()
    for e in range(E):
        r0, r1 = int(offs[e]), int(offs[e + 1])
        if r1 > r0:
            ref = oracle.gemm_w4a16(x[r0:r1], codes[e], exps[e])
            assert rel_l2(yh[r0:r1], ref) <= 2e-6, e


@pytest.mark.parametrize("G,mode", [(16, "channel"), (48, "token")])
def test_attention_many_query_rows_bench_shape(msd, G, mode):
    """The query-row sweep of bench.py at its size (B = 16, 8 KV heads, L = 4096) for the kernels that hold 16
    heads per pass: sampled batch entries against the oracle, per head."""
    B, Hkv, L, d = 16, 8, 4096, 128
    Hq = Hkv * G
    q = synth.queries(synth.seed_for(4, 100 + G), B, Hq, d)
    if mode == "token":
        Kc, ks, Vc, vs = synth.kv_cache_per_token(synth.seed_for(4, 7), B, Hkv, L, d)
        omode, gmode = oracle.PER_TOKEN, msd.MSD_PER_TOKEN
    else:
        Kc, ks, Vc, vs = synth.kv_cache_per_channel(synth.seed_for(4, 8), B, Hkv, L, d)
        omode, gmode = oracle.PER_CHANNEL, msd.MSD_PER_CHANNEL
    out = msd.msd_attn_decode_int8kv(bf16_to_dev(q), to_dev(Kc), to_dev(Vc), to_dev(ks), to_dev(vs), gmode)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert np.all(np.isfinite(o))
    sel = [0, 15]
    if mode == "token":
        ref = oracle.attn_decode(q[sel], Kc[sel], Vc[sel], ks[sel], vs[sel], omode)
    else:
        ref = oracle.attn_decode(q[sel], Kc[sel], Vc[sel], ks, vs, omode)
    for i, b in enumerate(sel):
        for h in range(Hq):
            assert rel_l2(o[b, h], ref[i, h]) <= 1e-3, (b, h)
