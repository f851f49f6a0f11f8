"""GPU parity of the decomposition-constant variants (paper Sec. 3.3: fractional INT8 scaling; the MXFP4
design-evolution table's v1 and v2; the E2M1-grid ablation) against the oracle's variants, through the C ABI, on every kernel
family.  Same bars as the main variant: codes, scales and int32 partials bit-exact, fp32 output within
1e-6 / 2e-6 relative L2."""
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


@pytest.mark.parametrize("M,K", [(1, 4096), (5, 48), (33, 8192), (3, 16400 - 16400 % 16)])
def test_decompose_int8_fractional_bit_exact(msd, M, K):
    x = synth.activations(synth.seed_for(5, M), M, K, outliers=K >= 1024)
    if M > 2:
        x[M // 2] = 0
    q1, q2, al, _ = oracle.decompose_int8(x, fractional=True)
    d1, d2, da = msd.msd_decompose_variant(msd.MSD_VARIANT_INT8_FRACTIONAL, msd.MSD_INT8, bf16_to_dev(x))
    torch.cuda.synchronize()
    assert np.array_equal(d1.cpu().numpy(), q1) and np.array_equal(d2.cpu().numpy(), q2)
    assert np.array_equal(da.cpu().numpy().view(np.uint32), al.view(np.uint32))
    m1, _, ma = oracle.decompose_int8(x)[:3]
    assert not np.array_equal(al, ma)                # the variant is a different quantiser


# fused single launch, skinny decode, wide decode, small and large asynchronous-fill tiles, K % 64 != 0
W8_SHAPES = [(1, 4096, 1024), (2, 1040, 300), (8, 4096, 512), (30, 512, 8300), (70, 320, 6500),
             (128, 256, 12800), (1100, 512, 4200), (300, 1040, 520)]


@pytest.mark.parametrize("M,K,N", W8_SHAPES)
@pytest.mark.parametrize("taps", [True, False])
def test_gemm_w8a16_fractional(msd, M, K, N, taps):
    seed = synth.seed_for(5, M * 13 + N)
    x = synth.activations(seed, M, K, outliers=True)
    W, s = synth.int8_weights(seed, N, K)
    xd, Wd, sd = bf16_to_dev(x), to_dev(W), to_dev(s)
    V = msd.MSD_VARIANT_INT8_FRACTIONAL
    if taps:
        y_ref, t = oracle.gemm_w8a16(x, W, s, fractional=True, taps=True)
        y, g = msd.msd_gemm_w8a16_variant(V, xd, Wd, sd, taps=True)
        torch.cuda.synchronize()
        for k in ("q1", "q2", "acc1", "acc2"):
            assert np.array_equal(g[k].cpu().numpy(), t[k]), k
        assert np.array_equal(g["scale"].cpu().numpy().view(np.uint32), t["alpha"].view(np.uint32))
    else:
        y_ref = oracle.gemm_w8a16(x, W, s, fractional=True)
        y = msd.msd_gemm_w8a16_variant(V, xd, Wd, sd)
        torch.cuda.synchronize()
    assert rel_l2(y.cpu().numpy(), y_ref) <= 1e-6
    # and the entry point without a variant still computes the main one
    y0 = msd.msd_gemm_w8a16(xd, Wd, sd)
    torch.cuda.synchronize()
    assert rel_l2(y0.cpu().numpy(), oracle.gemm_w8a16(x, W, s)) <= 1e-6


def _mx_variant(msd, variant):
    return {1: msd.MSD_VARIANT_MXFP4_V1, 2: msd.MSD_VARIANT_MXFP4_V2, 4: msd.MSD_VARIANT_MXFP4_E2M1}[variant]


@pytest.mark.parametrize("variant", [1, 2, 4])
@pytest.mark.parametrize("M,K", [(1, 4096), (7, 96), (40, 2048)])
def test_decompose_mxfp4_variants_bit_exact(msd, variant, M, K):
    x = synth.activations(synth.seed_for(6, M), M, K, outliers=K >= 1024)
    x[0, :32] = 0
    q1, q2, e = oracle.decompose_mxfp4(x, variant=variant)
    V = _mx_variant(msd, variant)
    d1, d2, de = msd.msd_decompose_variant(V, msd.MSD_MXFP4, bf16_to_dev(x))
    torch.cuda.synchronize()
    assert np.array_equal(d1.cpu().numpy(), q1) and np.array_equal(d2.cpu().numpy(), q2)
    assert np.array_equal(de.cpu().numpy(), e)


# fused single launch, stacked components (M <= 8), M <= 16, 32-row tiles, many rows (taps: the
# register-staged tile kernel; no taps: the asynchronous-fill kernel), K % 64 != 0
W4_SHAPES = [(1, 2048, 600), (2, 544, 300), (8, 1024, 520), (16, 512, 1000), (30, 512, 2100), (64, 512, 300),
             (100, 1024, 130), (200, 512, 700), (300, 544, 520), (90, 512, 260), (3, 512, 140)]


@pytest.mark.parametrize("variant", [1, 2, 4])
@pytest.mark.parametrize("M,K,N", W4_SHAPES)
@pytest.mark.parametrize("taps", [True, False])
def test_gemm_w4a16_variants(msd, variant, M, K, N, taps):
    seed = synth.seed_for(6, M * 13 + N)
    x = synth.activations(seed, M, K, outliers=True)
    codes, exps = synth.mxfp4_weights(seed, N, K)
    xd, cd, ed = bf16_to_dev(x), to_dev(codes), to_dev(exps)
    V = _mx_variant(msd, variant)
    if taps:
        y_ref, t = oracle.gemm_w4a16(x, codes, exps, variant=variant, taps=True)
        y, g = msd.msd_gemm_w4a16_variant(V, xd, cd, ed, taps=True)
        torch.cuda.synchronize()
        assert np.array_equal(g["q1"].cpu().numpy(), t["q1"])
        assert np.array_equal(g["q2"].cpu().numpy(), t["q2"])
        assert np.array_equal(g["scale"].cpu().numpy(), t["e8m0"])
    else:
        y_ref = oracle.gemm_w4a16(x, codes, exps, variant=variant)
        y = msd.msd_gemm_w4a16_variant(V, xd, cd, ed)
        torch.cuda.synchronize()
    assert rel_l2(y.cpu().numpy(), y_ref) <= 2e-6
    assert rel_l2(y.cpu().numpy(), oracle.gemm_w4a16(x, codes, exps)) > 1e-4      # not the main variant


def test_variant_must_belong_to_the_format(msd):
    x = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((8, 64), dtype=torch.int8, device="cuda")
    s = torch.ones(8, device="cuda")
    c = torch.zeros((8, 32), dtype=torch.uint8, device="cuda")
    e = torch.full((8, 2), 127, dtype=torch.uint8, device="cuda")
    for bad in (msd.MSD_VARIANT_MXFP4_V1, msd.MSD_VARIANT_MXFP4_V2, msd.MSD_VARIANT_MXFP4_E2M1, 9, -1):
        with pytest.raises(msd.MsdError) as err:
            msd.msd_gemm_w8a16_variant(bad, x, W, s)
        assert err.value.code == -1
        with pytest.raises(msd.MsdError) as err:
            msd.msd_decompose_variant(bad, msd.MSD_INT8, x)
        assert err.value.code == -1
    for bad in (msd.MSD_VARIANT_INT8_FRACTIONAL, 9):
        with pytest.raises(msd.MsdError) as err:
            msd.msd_gemm_w4a16_variant(bad, x, c, e)
        assert err.value.code == -1
        with pytest.raises(msd.MsdError) as err:
            msd.msd_decompose_variant(bad, msd.MSD_MXFP4, x)
        assert err.value.code == -1
    # MSD_VARIANT_MAIN is the entry point without a variant
    y0 = msd.msd_gemm_w8a16_variant(msd.MSD_VARIANT_MAIN, x, W, s)
    assert y0.shape == (4, 8)
