"""GPU parity of the grouped (mixture-of-experts) W8A16 GEMM against the oracle, through the C ABI.

Bar: fp32 output within 1e-6 relative L2 of the oracle per expert slice (the integer partial products are
those of msd_gemm_w8a16, whose kernel body the grouped kernel runs per expert and which is compared bit-exactly
elsewhere); rows that belong to no expert are not written."""
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


def _problem(seed, E, N, K, counts):
    T = int(sum(counts))
    x = synth.activations(seed, T, K, outliers=True)
    W = np.stack([synth.int8_weights(seed + 1 + e, N, K)[0] for e in range(E)])
    s = np.stack([synth.int8_weights(seed + 1 + e, N, K)[1] for e in range(E)])
    offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    return x, W, s, offs


CASES = [
    # E, N, K, rows per expert
    (4, 300, 512, [1, 0, 5, 2]),                 # an empty expert, ragged N
    (8, 128, 1024, [3, 1, 1, 0, 0, 8, 16, 2]),   # a full chunk of 16 rows
    (3, 520, 1040, [17, 40, 1]),                 # several chunks per expert, K not a multiple of 64
    (6, 64, 256, [0, 0, 0, 0, 0, 4]),            # all but one expert empty
    (2, 4096, 4096, [2, 7]),                     # decode-sized matrices
    (5, 330, 2048, [16, 0, 3, 9, 1]),            # row-segment weight loads (K a multiple of 2048), ragged N
]


@pytest.mark.parametrize("E,N,K,counts", CASES)
def test_moe_gemm_w8a16_parity(msd, E, N, K, counts):
    x, W, s, offs = _problem(synth.seed_for(8, E * 100 + N), E, N, K, counts)
    ref = oracle.moe_gemm_w8a16(x, offs, W, s)
    T = x.shape[0]
    y = torch.full((T, N), float("nan"), dtype=torch.float32, device="cuda")
    msd.msd_moe_gemm_w8a16(bf16_to_dev(x), to_dev(offs), to_dev(W), to_dev(s), y=y)
    torch.cuda.synchronize()
    yh = y.cpu().numpy()
    assert np.all(np.isfinite(yh))
    for e in range(E):
        r0, r1 = offs[e], offs[e + 1]
        if r1 > r0:
            assert rel_l2(yh[r0:r1], ref[r0:r1]) <= 1e-6
    # the same rows through the ungrouped entry point, expert by expert: identical bits
    for e in range(E):
        r0, r1 = int(offs[e]), int(offs[e + 1])
        if r1 > r0:
            ye = msd.msd_gemm_w8a16(bf16_to_dev(x[r0:r1]), to_dev(W[e]), to_dev(s[e]))
            assert np.array_equal(ye.cpu().numpy(), yh[r0:r1])


def test_moe_rows_without_expert_are_left_alone_and_bf16_output(msd):
    E, N, K = 3, 200, 512
    x, W, s, offs = _problem(5, E, N, K, [2, 3, 1])
    x = np.concatenate([x, x[:2]])                # two rows past expert_offsets[E]
    y = torch.full((8, N + 4), -7.0, dtype=torch.float32, device="cuda")
    msd.msd_moe_gemm_w8a16(bf16_to_dev(x), to_dev(offs), to_dev(W), to_dev(s), y=y[:, :N])
    torch.cuda.synchronize()
    yh = y.cpu().numpy()
    ref = oracle.moe_gemm_w8a16(x[:6], offs, W, s)
    assert rel_l2(yh[:6, :N], ref) <= 1e-6
    assert np.all(yh[6:] == -7.0) and np.all(yh[:, N:] == -7.0)
    yb = msd.msd_moe_gemm_w8a16(bf16_to_dev(x[:6]), to_dev(offs), to_dev(W), to_dev(s), out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert rel_l2(yb.float().cpu().numpy(), ref) <= 1e-2


def test_moe_error_codes(msd):
    x = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((2, 8, 64), dtype=torch.int8, device="cuda")
    s = torch.ones((2, 8), device="cuda")
    offs = torch.tensor([0, 2, 4], dtype=torch.int32, device="cuda")
    tiny = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(msd.MsdError) as e:
        msd.msd_moe_gemm_w8a16(x, offs, W, s, ws=tiny)
    assert e.value.code == -3
    y = msd.msd_moe_gemm_w8a16(x[:0], offs, W, s)     # no rows: a successful no-op
    assert y.shape == (0, 8)


W4_CASES = [
    (4, 300, 512, [1, 0, 5, 2]),                 # an empty expert, ragged N
    (8, 128, 1024, [3, 1, 1, 0, 0, 8, 16, 2]),   # one and two chunks of 8 rows
    (3, 520, 544, [17, 9, 1]),                   # several chunks, K not a multiple of 512
    (2, 4096, 4096, [2, 7]),                     # decode-sized matrices
]


@pytest.mark.parametrize("E,N,K,counts", W4_CASES)
def test_moe_gemm_w4a16_parity(msd, E, N, K, counts):
    seed = synth.seed_for(8, E * 100 + N + 1)
    T = int(sum(counts))
    x = synth.activations(seed, T, K, outliers=True)
    packs = [synth.mxfp4_weights(seed + 1 + e, N, K) for e in range(E)]
    codes = np.stack([p[0] for p in packs])
    exps = np.stack([p[1] for p in packs])
    offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    ref = oracle.moe_gemm_w4a16(x, offs, codes, exps)
    y = torch.full((T, N), float("nan"), dtype=torch.float32, device="cuda")
    msd.msd_moe_gemm_w4a16(bf16_to_dev(x), to_dev(offs), to_dev(codes), to_dev(exps), y=y)
    torch.cuda.synchronize()
    yh = y.cpu().numpy()
    assert np.all(np.isfinite(yh))
    for e in range(E):
        r0, r1 = offs[e], offs[e + 1]
        if r1 > r0:
            assert rel_l2(yh[r0:r1], ref[r0:r1]) <= 2e-6


def test_moe_offsets_past_the_last_row_are_clamped(msd):
    """A routing table whose last offset exceeds the number of rows must not take any row index out of the
    arrays: the kernels clamp it to T."""
    E, N, K = 2, 100, 512
    x, W, s, offs = _problem(11, E, N, K, [2, 3])
    bad = offs.copy()
    bad[-1] = 50
    y = msd.msd_moe_gemm_w8a16(bf16_to_dev(x), to_dev(bad), to_dev(W), to_dev(s))
    torch.cuda.synchronize()
    assert rel_l2(y.cpu().numpy(), oracle.moe_gemm_w8a16(x, offs, W, s)) <= 1e-6
