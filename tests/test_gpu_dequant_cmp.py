"""GPU parity of the comparison kernels (dequantise-then-BF16-MFMA) against the oracle's
dequant baseline (INT8) and the fp64 truth (MXFP4, whose lift to BF16 is exact)."""
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


@pytest.mark.parametrize("M,K,N", [(1, 4096, 512), (16, 1024, 1024), (32, 4096, 256), (70, 528, 100)])
def test_dequant_w8_matches_oracle_baseline(msd, M, K, N):
    x = synth.activations(61 + M, M, K)
    W, s = synth.int8_weights(61 + M, N, K)
    ref = oracle.dequant_gemm_w8a16(x, W, s)
    y = msd.msd_dequant_gemm_w8a16(bf16_to_dev(x), to_dev(W), to_dev(s))
    torch.cuda.synchronize()
    assert rel_l2(y.cpu().numpy(), ref) <= 1e-5
    # and it is the less accurate path: MSD is closer to the fp64 truth (Sec. 6.2); with 1 % outlier
    # channels x50 the row max grows and MSD's margin shrinks from ~200x to ~8x, so only 2x is asserted
    truth = oracle.truth_gemm_w8(x, W, s)
    y_msd = msd.msd_gemm_w8a16(bf16_to_dev(x), to_dev(W), to_dev(s))
    assert rel_l2(y_msd.cpu().numpy(), truth) * 2 < rel_l2(y.cpu().numpy(), truth)


@pytest.mark.parametrize("M,K,N", [(256, 512, 300), (300, 1056, 520), (700, 256, 777)])
def test_dequant_w8_two_step_form(msd, M, K, N):
    """M >= 256 with the full workspace: weights are written to HBM as BF16, then a tiled BF16 GEMM runs."""
    x = synth.activations(67 + M, M, K)
    W, s = synth.int8_weights(67 + M, N, K)
    ref = oracle.dequant_gemm_w8a16(x, W, s)
    xd, Wd, sd = bf16_to_dev(x), to_dev(W), to_dev(s)
    y = msd.msd_dequant_gemm_w8a16(xd, Wd, sd)
    torch.cuda.synchronize()
    assert rel_l2(y.cpu().numpy(), ref) <= 1e-5
    # the single-kernel form (no workspace) computes the same thing
    tiny = torch.empty(256, dtype=torch.uint8, device="cuda")
    y1 = msd.msd_dequant_gemm_w8a16(xd, Wd, sd, ws=tiny)
    torch.cuda.synchronize()
    assert rel_l2(y1.cpu().numpy(), ref) <= 1e-5


def test_dequant_w4_two_step_form(msd):
    M, K, N = 300, 544, 200
    x = synth.activations(73, M, K)
    codes, exps = synth.mxfp4_weights(73, N, K)
    truth = oracle.truth_gemm_w4(x, codes, exps)
    y = msd.msd_dequant_gemm_w4a16(bf16_to_dev(x), to_dev(codes), to_dev(exps))
    torch.cuda.synchronize()
    assert rel_l2(y.cpu().numpy(), truth) <= 1e-5


@pytest.mark.parametrize("M,K,N", [(1, 8192, 256), (32, 2048, 128), (40, 544, 72)])
def test_dequant_w4_matches_truth(msd, M, K, N):
    x = synth.activations(71 + M, M, K)
    codes, exps = synth.mxfp4_weights(71 + M, N, K)
    truth = oracle.truth_gemm_w4(x, codes, exps)
    y = msd.msd_dequant_gemm_w4a16(bf16_to_dev(x), to_dev(codes), to_dev(exps))
    torch.cuda.synchronize()
    assert rel_l2(y.cpu().numpy(), truth) <= 1e-5
