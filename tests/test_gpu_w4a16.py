"""GPU parity: msd_decompose (MXFP4) and msd_gemm_w4a16 against the CPU oracle, through the C ABI.

Bar: 4-bit component codes and E8M0 exponents bit-exact; fp32 output within relative L2 1e-3 of
the oracle (the GPU accumulates block products in fp32 inside the matrix instruction, the oracle
in fp64); Theorem-2 output bound against the fp64 truth."""
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


@pytest.mark.parametrize("M,K,scale", [(1, 8192, 1.0), (7, 96, 1e-3), (33, 4096, 300.0), (300, 544, 1.0)])
def test_decompose_mxfp4_bit_exact(msd, M, K, scale):
    x = synth.activations(synth.seed_for(3, M), M, K, outliers=K >= 1024, scale=scale)
    xf = synth.bf16_bits_to_f32(x).copy()
    xf[0, :32] = 0.0                       # all-zero block
    xf[M - 1, 32:64] = 0.0
    xf[M - 1, 33] = 1.859375               # equality case of the alpha rule
    xf[M - 1, 34] = 0.125                  # tie on the code grid
    x = synth.f32_to_bf16_bits(xf)
    q1, q2, e = oracle.decompose_mxfp4(x)
    d1, d2, de = msd.msd_decompose(msd.MSD_MXFP4, bf16_to_dev(x))
    torch.cuda.synchronize()
    assert np.array_equal(de.cpu().numpy(), e)
    assert np.array_equal(d1.cpu().numpy(), q1)
    assert np.array_equal(d2.cpu().numpy(), q2)


SHAPES = [(1, 8192, 512), (32, 8192, 256), (5, 96, 40), (17, 1056, 100), (70, 512, 48), (2, 2048, 4096),
          (200, 2048, 600), (130, 160, 300)]


@pytest.mark.parametrize("M,K,N", SHAPES)
def test_gemm_w4a16_parity(msd, M, K, N):
    seed = synth.seed_for(3, M * 11 + N)
    x = synth.activations(seed, M, K, outliers=K >= 1024)
    codes, exps = synth.mxfp4_weights(seed, N, K)
    y_ref, t = oracle.gemm_w4a16(x, codes, exps, taps=True)
    y, g = msd.msd_gemm_w4a16(bf16_to_dev(x), to_dev(codes), to_dev(exps), taps=True)
    torch.cuda.synchronize()
    assert np.array_equal(g["scale"].cpu().numpy(), t["e8m0"])
    assert np.array_equal(g["q1"].cpu().numpy(), t["q1"])
    assert np.array_equal(g["q2"].cpu().numpy(), t["q2"])
    yh = y.cpu().numpy()
    assert rel_l2(yh, y_ref) <= 1e-3
    assert rel_l2(yh, y_ref) <= 2e-6
    truth = oracle.truth_gemm_w4(x, codes, exps)
    a = np.exp2(t["e8m0"].astype(np.float64) - 127)
    wabs = np.abs(synth.dequantize_mxfp4(codes, exps).astype(np.float64)).reshape(N, -1, 32).sum(axis=2)
    bound = (a / 64) @ wabs.T
    assert np.all(np.abs(yh - truth) <= bound * (1 + 1e-5) + np.abs(truth) * 2.0 ** -20 + 1e-30)


@pytest.mark.parametrize("M,K,N", [(256, 512, 256), (300, 2048, 600), (40, 192, 70), (700, 64, 1000), (1, 8192, 512),
                                   (33, 4096, 300), (3, 512, 130), (4, 2048, 520), (3, 1024, 20000),
                                   # 9..32 rows with K a multiple of 512: weights straight to the matrix operand,
                                   # activation operands through LDS (one, two, three and many K batches)
                                   (32, 512, 128), (9, 1024, 300), (17, 1536, 1000), (32, 8192, 700), (24, 2048, 8300),
                                   # 33..128 rows: two or four 32-row groups, batches of four K steps
                                   (33, 512, 130), (64, 1024, 300), (100, 2048, 520), (128, 1536, 4200),
                                   (96, 1024, 300), (70, 2048, 520)])
def test_gemm_w4a16_product_path_without_taps(msd, M, K, N):
    """The path a caller without observation points takes: 3..128 rows with K a multiple of 512 go through
    the LDS-staged weight-stream kernel, more rows (or other K that is a multiple of 64) through the many-row
    pipeline (own operand format, transposed scale bytes, 256 x 256 tiles).  y starts as NaN and is computed
    twice."""
    seed = synth.seed_for(3, M * 13 + N)
    x = synth.activations(seed, M, K, outliers=K >= 1024)
    codes, exps = synth.mxfp4_weights(seed, N, K)
    y_ref = oracle.gemm_w4a16(x, codes, exps)
    y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    xd, cd, ed = bf16_to_dev(x), to_dev(codes), to_dev(exps)
    for _ in range(2):
        msd.msd_gemm_w4a16(xd, cd, ed, y=y)
        torch.cuda.synchronize()
        yh = y.cpu().numpy()
        assert np.all(np.isfinite(yh))
        assert rel_l2(yh, y_ref) <= 2e-6
    # BF16 output of the same path: RNE of the fp32 value
    yb = msd.msd_gemm_w4a16(xd, cd, ed, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert rel_l2(yb.float().cpu().numpy(), y_ref) <= 1e-2


@pytest.mark.parametrize("M,K,N", [(2, 1024, 256), (8, 512, 300), (100, 256, 300), (20, 1024, 300)])
def test_gemm_w4a16_strided_operands(msd, M, K, N):
    """ldx > K and ldy > N; pad columns of y stay untouched."""
    seed = synth.seed_for(3, M * 19 + N)
    x = synth.activations(seed, M, K)
    codes, exps = synth.mxfp4_weights(seed, N, K)
    y_ref = oracle.gemm_w4a16(x, codes, exps)
    xbig = torch.zeros((M, K + 40), dtype=torch.bfloat16, device="cuda")
    xbig[:, :K] = bf16_to_dev(x)
    ybig = torch.full((M, N + 5), -7.0, dtype=torch.float32, device="cuda")
    msd.msd_gemm_w4a16(xbig[:, :K], to_dev(codes), to_dev(exps), y=ybig[:, :N])
    torch.cuda.synchronize()
    yh = ybig.cpu().numpy()
    assert rel_l2(yh[:, :N], y_ref) <= 2e-6
    assert np.all(yh[:, N:] == -7.0)


def test_gemm_w4a16_bf16_out_and_errors(msd):
    M, K, N = 4, 1024, 64
    x = synth.activations(5, M, K)
    codes, exps = synth.mxfp4_weights(5, N, K)
    ref = oracle.gemm_w4a16(x, codes, exps, out_bf16=True)
    y = msd.msd_gemm_w4a16(bf16_to_dev(x), to_dev(codes), to_dev(exps), out_dtype=torch.bfloat16)
    bits = bf16_dev_to_bits(y)
    assert rel_l2(synth.bf16_bits_to_f32(bits), synth.bf16_bits_to_f32(ref)) <= 1e-3
    assert np.mean(bits != ref) < 0.01
    with pytest.raises(msd.MsdError) as e:
        msd.msd_gemm_w4a16(torch.zeros((2, 48), dtype=torch.bfloat16, device="cuda"),
                           torch.zeros((4, 24), dtype=torch.uint8, device="cuda"),
                           torch.zeros((4, 1), dtype=torch.uint8, device="cuda"))
    assert e.value.code == -2


PACKED_SHAPES = [
    (1, 8192, 512), (1, 512, 40), (2, 2048, 4096), (3, 1024, 300), (4, 512, 8300),          # register-operand kernel
    (9, 1024, 300), (32, 8192, 700), (24, 2048, 8300), (64, 1024, 300), (128, 1536, 4200),  # LDS-staged weight stream
    (1, 1024, 12400), (2, 512, 17590), (2, 1536, 20000), (1, 2560, 28672), (1, 512, 40000), (2, 16384, 20000), (4, 512, 28672),
    # one or two rows, many channels: the single-launch kernel with 4..8 tiles per workgroup, a ragged last tile,
    # two rounds, K ranges that do not split evenly into four parts, more than two blocks per thread; four rows
    # on the same channels stay on the two-launch form
    (24, 512, 17590), (32, 1024, 28672),   # up to 32 rows, many channels (more workgroups than CUs)
    (16, 1024, 17590), (11, 512, 28672), (5, 8192, 300), (13, 1536, 40),   # up to 16 rows: the half-size operand image
    (40, 512, 700), (64, 8192, 300), (100, 1024, 17590), (128, 512, 40),   # 33..128 rows: two and four row groups
    (65, 1024, 300), (96, 512, 17590), (80, 8192, 140),                     # 65..96 rows: three row groups
    (256, 512, 256), (300, 2048, 600), (700, 512, 1000),                                     # many-row pipeline
]


@pytest.mark.parametrize("M,K,N", PACKED_SHAPES)
def test_gemm_w4a16_packed_weights(msd, M, K, N):
    """msd_gemm_w4a16_packed against the oracle (which reads the canonical layout) and bit-identical to
    msd_gemm_w4a16 on the canonical arrays (same instructions on the same operands, another address map)."""
    seed = synth.seed_for(3, M * 17 + N)
    x = synth.activations(seed, M, K, outliers=K >= 1024)
    codes, exps = synth.mxfp4_weights(seed, N, K)
    y_ref = oracle.gemm_w4a16(x, codes, exps)
    xd, cd, ed = bf16_to_dev(x), to_dev(codes), to_dev(exps)
    Wp, Ep = msd.msd_pack_weights_w4(cd, ed)
    y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    msd.msd_gemm_w4a16_packed(xd, Wp, Ep, N, y=y)
    torch.cuda.synchronize()
    yh = y.cpu().numpy()
    assert np.all(np.isfinite(yh))
    assert rel_l2(yh, y_ref) <= 2e-6
    assert torch.equal(y, msd.msd_gemm_w4a16(xd, cd, ed))
    if M <= 16:  # observation points ride on the register-operand kernel
        y2, g = msd.msd_gemm_w4a16_packed(xd, Wp, Ep, N, taps=True)
        torch.cuda.synchronize()
        _, t = oracle.gemm_w4a16(x, codes, exps, taps=True)
        assert np.array_equal(g["q1"].cpu().numpy(), t["q1"]) and np.array_equal(g["q2"].cpu().numpy(), t["q2"])
        assert np.array_equal(g["scale"].cpu().numpy(), t["e8m0"])
        assert rel_l2(y2.cpu().numpy(), y_ref) <= 2e-6


@pytest.mark.parametrize("M,K,N,shift", [(1, 1024, 13000, 3), (2, 512, 17590, 8), (2, 1536, 12400, 1)])
def test_gemm_w4a16_packed_single_launch_strided(msd, M, K, N, shift):
    """The single-launch kernel for one or two rows on packed weights with ldx > K, rows of x that are not
    16-byte aligned (shift not a multiple of 8 elements), ldy > N, and BF16 output: equal to the canonical entry
    point bit for bit, pad columns untouched."""
    seed = synth.seed_for(3, M * 23 + N)
    x = synth.activations(seed, M, K, outliers=True)
    codes, exps = synth.mxfp4_weights(seed, N, K)
    y_ref = oracle.gemm_w4a16(x, codes, exps)
    cd, ed = to_dev(codes), to_dev(exps)
    Wp, Ep = msd.msd_pack_weights_w4(cd, ed)
    xbig = torch.zeros((M, K + 40), dtype=torch.bfloat16, device="cuda")
    xv = xbig[:, shift:shift + K]
    xv.copy_(bf16_to_dev(x))
    ybig = torch.full((M, N + 5), -7.0, dtype=torch.float32, device="cuda")
    msd.msd_gemm_w4a16_packed(xv, Wp, Ep, N, y=ybig[:, :N])
    torch.cuda.synchronize()
    yh = ybig.cpu().numpy()
    assert rel_l2(yh[:, :N], y_ref) <= 2e-6
    assert np.all(yh[:, N:] == -7.0)
    assert torch.equal(ybig[:, :N], msd.msd_gemm_w4a16(bf16_to_dev(x), cd, ed))
    yb = msd.msd_gemm_w4a16_packed(xv, Wp, Ep, N, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert torch.equal(yb, msd.msd_gemm_w4a16(bf16_to_dev(x), cd, ed, out_dtype=torch.bfloat16))


def test_pack_weights_w4_layout_and_errors(msd):
    """The packed arrays are exactly the documented permutations (zero / 0x7F padding past N); K % 512 != 0 is refused."""
    N, K = 40, 1024
    codes, exps = synth.mxfp4_weights(synth.seed_for(3, 99), N, K)
    Wp, Ep = msd.msd_pack_weights_w4(to_dev(codes), to_dev(exps))
    torch.cuda.synchronize()
    tiles = (N + 15) // 16
    want = np.zeros((K // 128, tiles, 4, 16, 16), dtype=np.uint8)       # [q][nb][g][r][b]
    cp = np.zeros((tiles * 16, K // 32, 16), dtype=np.uint8)
    cp[:N] = codes.reshape(N, K // 32, 16)
    for q in range(K // 128):
        for g in range(4):
            want[q, :, g] = cp[:, 4 * q + g].reshape(tiles, 16, 16)
    assert np.array_equal(Wp.cpu().numpy(), want.reshape(-1))
    ep = np.full((tiles * 16, K // 32), 0x7F, dtype=np.uint8)
    ep[:N] = exps
    want_e = ep.reshape(tiles, 16, K // 512, 16).transpose(2, 0, 1, 3)   # [s][nb][r][i]
    Eh = Ep.cpu().numpy()
    assert np.array_equal(Eh[:want_e.size], want_e.reshape(-1))
    # second part (256-byte aligned): the same bytes per K step of 64 and tile of 256 channels, channel r of the
    # tile and block b of the step at (r // 128) * 256 + b * 128 + (r % 32) * 4 + (r // 32) % 4; 0x7F past N
    first = (want_e.size + 255) // 256 * 256
    npad = (N + 255) // 256 * 256
    e2 = np.full((npad, K // 32), 0x7F, dtype=np.uint8)
    e2[:N] = exps
    want_t = np.zeros((K // 64, npad // 256, 512), dtype=np.uint8)
    r = np.arange(256)
    for b in range(2):
        slot = (r // 128) * 256 + b * 128 + (r % 32) * 4 + (r // 32) % 4
        want_t[:, :, slot] = e2[:, b::2].reshape(npad // 256, 256, K // 64).transpose(2, 0, 1)
    assert np.array_equal(Eh[first:], want_t.reshape(-1))
    L = msd.lib()
    assert L.msd_packed_weights_w4_bytes(N, K) == want.size and L.msd_packed_scales_w4_bytes(N, K) == first + want_t.size
    assert L.msd_packed_weights_w4_bytes(0, K) == 0
    bad = L.msd_pack_weights_w4(Wp.data_ptr(), Ep.data_ptr(), N, 544, Wp.data_ptr(), Ep.data_ptr(), None)
    assert bad == -2  # MSD_ERR_SHAPE
