"""GPU parity: msd_decompose (INT8) and msd_gemm_w8a16 against the CPU oracle, through the C ABI.

Bar: INT8 codes, alpha bits and both int32 partial products bit-exact; fp32 output within
relative L2 1e-3 of the oracle (the stated bar) and, tighter, 1e-6 (the epilogue differs from
the oracle's fp64 merge only by a handful of fp32 roundings); Theorem-1 output bound against
the fp64 truth."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_13915_amd import synth
from gpu_util import bf16_to_dev, to_dev, rel_l2, bf16_dev_to_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def msd():
    from paper_2605_13915_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("M,K", [(1, 4096), (16, 1024), (5, 48), (3, 16400), (33, 8192), (7, 70000)])
def test_decompose_int8_bit_exact(msd, M, K):
    K = K - K % 16
    x = synth.activations(synth.seed_for(0, M), M, K, outliers=K >= 1024)
    x[M // 2, :] = 0 if M > 2 else x[M // 2, :]          # an all-zero row
    q1, q2, al, be = oracle.decompose_int8(x)
    d1, d2, da = msd.msd_decompose(msd.MSD_INT8, bf16_to_dev(x))
    torch.cuda.synchronize()
    assert np.array_equal(d1.cpu().numpy(), q1)
    assert np.array_equal(d2.cpu().numpy(), q2)
    assert np.array_equal(da.cpu().numpy().view(np.uint32), al.view(np.uint32))


def test_decompose_int8_every_bf16_value_under_many_scales(msd):
    """The division-free quantiser against the oracle's divisions, exhaustively: every finite BF16 value of
    either sign that does not exceed the row maximum, for row maxima sweeping all 128 BF16 significands in
    three binades (powers of two and their neighbours included, where x/alpha is an exact rounding tie for
    many x), both range-constant variants."""
    pats = np.arange(0x0000, 0x7F80, dtype=np.uint16)          # every non-negative finite BF16 pattern
    K = 65536
    rows = []
    for e in (121, 127, 131):
        for m in range(128):
            mx = np.uint16((e << 7) | m)
            vals = pats[pats <= mx]
            row = np.zeros(K, np.uint16)
            row[:len(vals)] = vals
            row[len(vals):2 * len(vals)] = vals | np.uint16(0x8000)
            rows.append(row)
    x = np.stack(rows)
    xd = bf16_to_dev(x)
    for frac in (False, True):
        q1, q2, al, _ = oracle.decompose_int8(x, fractional=frac)
        if frac:
            d1, d2, da = msd.msd_decompose_variant(msd.MSD_VARIANT_INT8_FRACTIONAL, msd.MSD_INT8, xd)
        else:
            d1, d2, da = msd.msd_decompose(msd.MSD_INT8, xd)
        torch.cuda.synchronize()
        assert np.array_equal(da.cpu().numpy().view(np.uint32), al.view(np.uint32))
        assert np.array_equal(d1.cpu().numpy(), q1)
        assert np.array_equal(d2.cpu().numpy(), q2)


def test_decompose_strided_rows(msd):
    x = synth.activations(3, 6, 512)
    big = torch.zeros((6, 520), dtype=torch.bfloat16, device="cuda")
    big[:, :512] = bf16_to_dev(x)
    d1, d2, da = msd.msd_decompose(msd.MSD_INT8, big[:, :512])      # ldx = 520 (16-byte aligned rows)
    odd = torch.zeros((6, 515), dtype=torch.bfloat16, device="cuda")
    odd[:, :512] = bf16_to_dev(x)
    e1, e2, ea = msd.msd_decompose(msd.MSD_INT8, odd[:, :512])      # ldx = 515: unaligned path
    q1, q2, al, _ = oracle.decompose_int8(x)
    for a, b in ((d1, q1), (d2, q2), (e1, q1), (e2, q2)):
        assert np.array_equal(a.cpu().numpy(), b)
    assert np.array_equal(da.cpu().numpy(), al) and np.array_equal(ea.cpu().numpy(), al)


SHAPES = [
    (16, 1024, 1024, 0),       # config 0
    (1, 4096, 4096, 1), (8, 4096, 4096, 1), (8, 4096, 8300, 1),   # decode: single launch; two launches, skinny kernel
    (5, 4096, 1000, 0), (4, 8192, 520, 1),   # just above the single-launch bound
    (32, 4096, 4096, 1),       # decode, split-K tiled kernel
    (3, 208, 50, 0),           # ragged everything, K not a multiple of 64
    (40, 1040, 200, 1),        # ragged tiled, several M tiles
    (130, 512, 300, 1),        # larger-tile kernel with ragged tails
    (128, 4096, 1024, 1),
    (300, 1040, 520, 1),       # several large tiles, ragged in M, N and K
    (257, 256, 777, 0),
    (1100, 512, 4200, 1),      # >= 128 large tiles: the asynchronous-LDS-fill kernel, ragged M and N
    (128, 256, 12800, 1),      # batched decode, 64x128 tiles of the asynchronous-fill kernel
    (70, 320, 6500, 1),        # batched decode, 64x64 tiles, ragged M and N
    (30, 512, 8300, 1),        # 16 < M <= 32 with many columns: 32x64 tiles of the asynchronous-fill kernel
    (32, 528, 8300, 0),        # same M and N, K not a multiple of 64: register-operand kernel, wide variant
    # 32x64 tiles on eight waves in four K groups (at most 256 tiles, K % 128 == 0): ragged M and N, fewer K
    # stages than the pipeline is deep, one stage more than that
    (64, 1024, 4100, 1), (100, 256, 1000, 1), (33, 640, 2000, 0),
    # the single-launch kernel with every load in flight at once (M*K <= 16384), one case per instance
    (4, 4096, 4096, 1), (3, 4096, 1000, 1),   # 4 waves x 16 K steps
    (2, 4096, 8300, 1),        # many column tiles, two per workgroup
    (4, 4096, 8300, 1),        # many column tiles, 8 waves x 8 steps, four tiles per workgroup
    (8, 2048, 530, 1), (5, 2048, 8300, 0),   # 4 x 8
    (8, 1024, 90, 1),          # 4 x 4 with 8 rows
    (13, 1024, 90, 1), (9, 1024, 1030, 0), (9, 2048, 90, 1),   # more rows than the row bound: two launches
    (2, 8192, 300, 1), (1, 8192, 8300, 1),   # 8 x 16, one and two tiles per workgroup
]


@pytest.mark.parametrize("M,K,N,outl", SHAPES)
def test_gemm_w8a16_parity(msd, M, K, N, outl):
    seed = synth.seed_for(1, M * 7 + N)
    x = synth.activations(seed, M, K, outliers=bool(outl))
    W, s = synth.int8_weights(seed, N, K)
    y_ref, t = oracle.gemm_w8a16(x, W, s, taps=True)
    y, g = msd.msd_gemm_w8a16(bf16_to_dev(x), to_dev(W), to_dev(s), taps=True)
    torch.cuda.synchronize()
    assert np.array_equal(g["q1"].cpu().numpy(), t["q1"])
    assert np.array_equal(g["q2"].cpu().numpy(), t["q2"])
    assert np.array_equal(g["scale"].cpu().numpy().view(np.uint32), t["alpha"].view(np.uint32))
    assert np.array_equal(g["acc1"].cpu().numpy(), t["acc1"])
    assert np.array_equal(g["acc2"].cpu().numpy(), t["acc2"])
    yh = y.cpu().numpy()
    assert rel_l2(yh, y_ref) <= 1e-3
    assert rel_l2(yh, y_ref) <= 1e-6
    # accuracy bound against the fp64 truth (Theorem 1 pushed through the dot product)
    truth = oracle.truth_gemm_w8(x, W, s)
    xf = synth.bf16_bits_to_f32(x).astype(np.float64)
    bound = s.astype(np.float64)[None] * np.abs(W.astype(np.float64)).sum(1)[None] * np.abs(xf).max(1)[:, None] / 64516.0
    assert np.all(np.abs(yh - truth) <= bound * (1 + 1e-4) + np.abs(truth) * 2.0 ** -21 + 1e-30)


@pytest.mark.parametrize("M,K,N", [(128, 4096, 1024), (100, 1024, 700), (96, 2112, 520), (65, 192, 300),
                                   (128, 4096, 14336 // 4), (1, 4096, 1024), (2, 1040, 300), (8, 4096, 512),
                                   # fragment-major codes (register-operand kernels): 1, 2 and 4 fragments, few and
                                   # many column tiles, K with a partial last batch of steps, ragged N
                                   (5, 4096, 8300), (8, 4096, 4096), (16, 4096, 4100), (12, 2112, 700),
                                   (32, 4096, 4096), (27, 4096, 1000), (9, 64, 20), (15, 8192, 8300),
                                   (20, 1088, 333), (6, 16384, 520), (24, 4096, 4096), (18, 2112, 260),
                                   # single-launch kernel without observation points
                                   (4, 4096, 4096), (16, 1024, 1024), (7, 2048, 8300), (2, 8192, 4000)])
def test_gemm_w8a16_product_path_without_taps(msd, M, K, N):
    """The path a caller without observation points takes.  y starts as NaN."""
    seed = synth.seed_for(1, M * 11 + N)
    x = synth.activations(seed, M, K, outliers=True)
    if M >= 3:
        x[1, :] = 0      # an all-zero row between the others
    W, s = synth.int8_weights(seed, N, K)
    y_ref = oracle.gemm_w8a16(x, W, s)
    y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    xd, Wd, sd = bf16_to_dev(x), to_dev(W), to_dev(s)
    for _ in range(2):      # a second call over its own previous result
        msd.msd_gemm_w8a16(xd, Wd, sd, y=y)
        torch.cuda.synchronize()
        yh = y.cpu().numpy()
        assert np.all(np.isfinite(yh))
        assert rel_l2(yh, y_ref) <= 1e-6


@pytest.mark.parametrize("M,K,N", [(2, 1024, 256), (8, 512, 300), (24, 256, 8300), (100, 256, 700), (300, 512, 600)])
def test_gemm_w8a16_strided_operands_and_bf16_output(msd, M, K, N):
    """Row strides larger than the row length for x and y (ldx > K, ldy > N; the pad columns of y must stay
    untouched), on every kernel family; then BF16 output of the same call."""
    seed = synth.seed_for(1, M * 17 + N)
    x = synth.activations(seed, M, K, outliers=True)
    W, s = synth.int8_weights(seed, N, K)
    y_ref = oracle.gemm_w8a16(x, W, s)
    xbig = torch.zeros((M, K + 24), dtype=torch.bfloat16, device="cuda")
    xbig[:, :K] = bf16_to_dev(x)
    ybig = torch.full((M, N + 9), -7.0, dtype=torch.float32, device="cuda")
    Wd, sd = to_dev(W), to_dev(s)
    msd.msd_gemm_w8a16(xbig[:, :K], Wd, sd, y=ybig[:, :N])
    torch.cuda.synchronize()
    yh = ybig.cpu().numpy()
    assert rel_l2(yh[:, :N], y_ref) <= 1e-6
    assert np.all(yh[:, N:] == -7.0)
    yb = msd.msd_gemm_w8a16(xbig[:, :K], Wd, sd, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    ref_bits = oracle.gemm_w8a16(x, W, s, out_bf16=True)
    bits = bf16_dev_to_bits(yb)
    assert np.mean(bits != ref_bits) < 0.01          # equal up to rare one-ulp ties of nearly equal fp32 values
    assert rel_l2(synth.bf16_bits_to_f32(bits), synth.bf16_bits_to_f32(ref_bits)) <= 1e-3


def test_gemm_w8a16_bf16_output_and_determinism(msd):
    M, K, N = 8, 1024, 512
    x = synth.activations(77, M, K)
    W, s = synth.int8_weights(77, N, K)
    ref = oracle.gemm_w8a16(x, W, s, out_bf16=True)
    xd, Wd, sd = bf16_to_dev(x), to_dev(W), to_dev(s)
    y = msd.msd_gemm_w8a16(xd, Wd, sd, out_dtype=torch.bfloat16)
    y2 = msd.msd_gemm_w8a16(xd, Wd, sd, out_dtype=torch.bfloat16)
    bits = bf16_dev_to_bits(y)
    assert np.array_equal(bits, bf16_dev_to_bits(y2))
    a = synth.bf16_bits_to_f32(bits)
    b = synth.bf16_bits_to_f32(ref)
    assert rel_l2(a, b) <= 1e-3
    # BF16 rounding of nearly equal fp32 values: at most one ulp apart, and only rarely
    assert np.mean(bits != ref) < 0.01


def test_gemm_w8a16_error_codes(msd):
    x = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((8, 64), dtype=torch.int8, device="cuda")
    s = torch.ones(8, device="cuda")
    tiny = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(msd.MsdError) as e:
        msd.msd_gemm_w8a16(x, W, s, ws=tiny)
    assert e.value.code == -3
    x2 = torch.zeros((4, 24), dtype=torch.bfloat16, device="cuda")
    W2 = torch.zeros((8, 24), dtype=torch.int8, device="cuda")
    with pytest.raises(msd.MsdError) as e:
        msd.msd_gemm_w8a16(x2, W2, s)
    assert e.value.code == -2
    # empty problems are successful no-ops
    y = msd.msd_gemm_w8a16(x[:0], W, s)
    assert y.shape == (0, 8)


def test_measurement_aids_run(msd):
    """msd_stream_read and msd_probe_mfma_w8a16 compute nothing that can be checked; they must run, leave
    their inputs alone and reject shapes they do not support."""
    W = torch.randint(-127, 128, (300, 512), dtype=torch.int8, device="cuda")
    W0 = W.clone()
    msd.msd_stream_read(W)
    msd.msd_stream_read_linear(W)                        # 153600 bytes: two workgroups and a ragged tail
    msd.msd_stream_read_linear(W.view(-1)[:48])
    assert msd.lib().msd_stream_read_linear(W.data_ptr(), 40, None) == -2   # not a multiple of 16
    ops = torch.randint(-2 ** 31, 2 ** 31 - 1, (16384,), dtype=torch.int32, device="cuda")
    assert msd.msd_probe_mfma_rate(msd.MSD_INT8, ops, 3) == 2048 * 8 * 3 * 65536
    assert msd.msd_probe_mfma_rate(msd.MSD_MXFP4, ops, 0) == 0
    assert msd.lib().msd_probe_mfma_rate(7, ops.data_ptr(), 1, None) == -1
    # LDS fill probe: window and stream of one kilobyte each (every address wraps), no rounds, a few rounds
    small = W.view(-1)[:2048]
    assert msd.msd_probe_lds_fill_rate(small, 1024, 2, 5) == 256 * 5 * 32768
    assert msd.msd_probe_lds_fill_rate(W.view(-1)[:153600], 4096, 4, 0) == 0
    assert msd.msd_probe_lds_fill_rate(W.view(-1)[:153600], 4096, 0, 3) == 256 * 3 * 32768
    assert msd.lib().msd_probe_lds_fill_rate(W.data_ptr(), 2048, 2048, 2, 1, None) == -2   # no stream part
    assert msd.lib().msd_probe_lds_fill_rate(W.data_ptr(), 4096, 1024, 5, 1, None) == -2   # hot_parts > 4
    assert msd.lib().msd_probe_lds_fill_rate(W.data_ptr(), 4000, 1024, 1, 1, None) == -2   # not whole kilobytes
    assert msd.lib().msd_probe_lds_fill_rate(None, 4096, 1024, 1, 1, None) == -1
    x = bf16_to_dev(synth.activations(5, 300, 512))
    s = torch.rand(300, device="cuda")
    y = msd.msd_probe_mfma_w8a16(x, W, s)
    torch.cuda.synchronize()
    assert y.shape == (300, 300) and torch.equal(W, W0)
    with pytest.raises(msd.MsdError) as e:
        msd.msd_probe_mfma_w8a16(x[:, :48].contiguous(), W[:, :48].contiguous(), s)
    assert e.value.code == -2
    with pytest.raises(msd.MsdError) as e:
        msd.msd_stream_read(W[:, :100].contiguous())
    assert e.value.code == -2
    codes, exps = synth.mxfp4_weights(9, 300, 512)
    y4 = msd.msd_probe_mfma_w4a16(x, to_dev(codes), to_dev(exps))
    torch.cuda.synchronize()
    assert y4.shape == (300, 300)
    with pytest.raises(msd.MsdError) as e:      # 32 rows or fewer never reach the many-row kernel
        msd.msd_probe_mfma_w4a16(x[:8], to_dev(codes), to_dev(exps))
    assert e.value.code == -2


def test_gemm_w8a16_maximum_k_extremal_codes(msd):
    """K = 131072, the largest accepted contraction length, with every code at +-127: the int32 partial
    products sit 1.6 % below 2^31 and must come out exactly, on the single-launch path (M = 1), the
    register-operand decode path (M = 3) and with observation points."""
    K, N = 131072, 33
    W = np.full((N, K), 127, np.int8)
    W[1::2] = -127
    s = np.linspace(0.5, 1.5, N).astype(np.float32)
    for M in (1, 3):
        vals = np.full((M, K), 3.0, np.float32)
        vals[M - 1] = -0.75
        x = synth.f32_to_bf16_bits(vals)
        y_ref, t = oracle.gemm_w8a16(x, W, s, taps=True)
        assert not t["overflow"] and abs(int(t["acc1"][0, 0])) == 127 * 127 * K
        y, g = msd.msd_gemm_w8a16(bf16_to_dev(x), to_dev(W), to_dev(s), taps=True)
        torch.cuda.synchronize()
        assert np.array_equal(g["acc1"].cpu().numpy(), t["acc1"])
        assert np.array_equal(g["acc2"].cpu().numpy(), t["acc2"])
        assert rel_l2(y.cpu().numpy(), y_ref) <= 1e-6
        y2 = msd.msd_gemm_w8a16(bf16_to_dev(x), to_dev(W), to_dev(s))
        torch.cuda.synchronize()
        assert rel_l2(y2.cpu().numpy(), y_ref) <= 1e-6
    with pytest.raises(msd.MsdError) as e:      # one chunk more is a shape error, not an overflow
        msd.msd_gemm_w8a16(torch.zeros((1, K + 16), dtype=torch.bfloat16, device="cuda"),
                           torch.zeros((N, K + 16), dtype=torch.int8, device="cuda"), to_dev(s))
    assert e.value.code == -2


@pytest.mark.parametrize("ex", [-130, -125, -118, -100, 100, 126])
def test_extreme_magnitudes_stay_bit_exact(msd, ex):
    """Rows whose scale beta (or alpha) is a denormal fp32 number, and rows near the top of the BF16 range:
    codes and alpha must still be those of correctly rounded fp32 division (the reciprocal shortcut of the
    quantiser does not apply there), in the stand-alone decomposition, the single-launch GEMM (M = 1) and the
    two-launch GEMM (M = 4)."""
    rng = np.random.default_rng(1000 + ex)
    vals = rng.standard_normal((4, 256)).astype(np.float32) * np.float32(2.0) ** ex
    x = synth.f32_to_bf16_bits(vals)
    q1, q2, al, _ = oracle.decompose_int8(x)
    d1, d2, da = msd.msd_decompose(msd.MSD_INT8, bf16_to_dev(x))
    torch.cuda.synchronize()
    assert np.array_equal(d1.cpu().numpy(), q1) and np.array_equal(d2.cpu().numpy(), q2)
    assert np.array_equal(da.cpu().numpy().view(np.uint32), al.view(np.uint32))
    W, s = synth.int8_weights(7, 40, 256)
    for M in (1, 4):
        _, t = oracle.gemm_w8a16(x[:M], W, s, taps=True)
        _, g = msd.msd_gemm_w8a16(bf16_to_dev(x[:M]), to_dev(W), to_dev(s), taps=True)
        torch.cuda.synchronize()
        for k in ("q1", "q2", "acc1", "acc2"):
            assert np.array_equal(g[k].cpu().numpy(), t[k]), (M, k)
    m1, m2, me = oracle.decompose_mxfp4(x)
    g1, g2, ge = msd.msd_decompose(msd.MSD_MXFP4, bf16_to_dev(x))
    torch.cuda.synchronize()
    assert np.array_equal(g1.cpu().numpy(), m1) and np.array_equal(g2.cpu().numpy(), m2)
    assert np.array_equal(ge.cpu().numpy(), me)


# ---------------------------------------------------------------- packed weights (msd_pack_weights_w8)
PACKED_SHAPES = [
    (1, 4096, 4096), (2, 4096, 8300), (4, 2048, 530), (8, 1024, 90), (3, 8192, 300),        # single-launch kernel
    (4, 4096, 9000), (2, 8192, 8400), (1, 2048, 8200),   # ... many column tiles: row-segment loads on the canonical layout
    (8, 4096, 4096), (5, 4096, 8300), (16, 4096, 4100), (12, 2112, 700), (32, 4096, 1000),  # register-operand kernels
    (15, 8192, 8300), (9, 64, 20), (20, 4096, 4100), (24, 1024, 90), (17, 2112, 700),   # ... 17..24 rows: three fragments
    (30, 512, 8300), (70, 320, 6500), (128, 256, 12800), (128, 4096, 1024), (100, 1024, 700),   # small LDS tiles
    (65, 192, 300), (96, 2112, 520), (64, 1024, 4100), (100, 256, 1000), (33, 640, 2000), (128, 128, 640),
    (48, 512, 4096), (64, 256, 3000), (40, 1024, 4000),   # at most 128 tiles of 32 x 64: the 32 x 32 tile instance
    (1100, 512, 4200), (300, 1088, 520), (257, 256, 777),                                    # large LDS tiles
]


@pytest.mark.parametrize("M,K,N", PACKED_SHAPES)
def test_gemm_w8a16_packed_weights(msd, M, K, N):
    """msd_gemm_w8a16_packed against the oracle (which reads the canonical layout), with and without
    observation points: integer partial products bit-exact, outputs within 1e-6, and bit-identical to
    msd_gemm_w8a16 on the canonical weights (same kernels, same arithmetic, another address map)."""
    seed = synth.seed_for(1, M * 13 + N)
    x = synth.activations(seed, M, K, outliers=True)
    if M >= 3:
        x[1, :] = 0
    W, s = synth.int8_weights(seed, N, K)
    y_ref, t = oracle.gemm_w8a16(x, W, s, taps=True)
    xd, Wd, sd = bf16_to_dev(x), to_dev(W), to_dev(s)
    Wp = msd.msd_pack_weights_w8(Wd)
    y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    msd.msd_gemm_w8a16_packed(xd, Wp, sd, y=y)
    torch.cuda.synchronize()
    yh = y.cpu().numpy()
    assert np.all(np.isfinite(yh))
    assert rel_l2(yh, y_ref) <= 1e-6
    for m in range(M):
        assert rel_l2(yh[m], y_ref[m]) <= 1e-6 or not np.any(y_ref[m]), m
    assert torch.equal(y, msd.msd_gemm_w8a16(xd, Wd, sd))
    y2, g = msd.msd_gemm_w8a16_packed(xd, Wp, sd, taps=True)
    torch.cuda.synchronize()
    assert np.array_equal(g["q1"].cpu().numpy(), t["q1"]) and np.array_equal(g["q2"].cpu().numpy(), t["q2"])
    assert np.array_equal(g["acc1"].cpu().numpy(), t["acc1"]) and np.array_equal(g["acc2"].cpu().numpy(), t["acc2"])
    assert rel_l2(y2.cpu().numpy(), y_ref) <= 1e-6


def test_pack_weights_layout_and_errors(msd):
    """The packed array is exactly the documented permutation of W (zero padding past N); K % 64 != 0 is refused."""
    N, K = 37, 192
    W = torch.randint(-127, 128, (N, K), dtype=torch.int8, device="cuda")
    P = msd.msd_pack_weights_w8(W).cpu().numpy().reshape(K // 64, (N + 15) // 16, 4, 16, 16)
    Wn = np.zeros(((N + 15) // 16 * 16, K), np.int8)
    Wn[:N] = W.cpu().numpy()
    ref = Wn.reshape((N + 15) // 16, 16, K // 64, 4, 16).transpose(2, 0, 3, 1, 4)   # [ks][nb][g][r][b]
    assert np.array_equal(P, ref)
    with pytest.raises(msd.MsdError) as e:
        msd.msd_pack_weights_w8(torch.zeros((16, 48), dtype=torch.int8, device="cuda"))
    assert e.value.code == -2
