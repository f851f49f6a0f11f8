"""msd_gemm_w8a16_static (built-in scratch buffer, no allocation) against msd_gemm_w8a16."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2605_13915_amd import binding as msd, synth
from gpu_util import bf16_to_dev, to_dev

pytestmark = pytest.mark.gpu


def _case(seed, M, K, N):
    x = bf16_to_dev(synth.activations(seed, M, K, outliers=True))
    W, s = synth.int8_weights(seed + 1, N, K)
    return x, to_dev(W), to_dev(s)


@pytest.mark.parametrize("shapes", [
    [(128, 4096, 1024), (8, 1024, 512)],      # asynchronous-fill kernel (blocked codes), then the register-operand kernel
    [(32, 2048, 4096), (1, 4096, 768)],       # two launches, then the single-launch form (scratch untouched)
    [(40, 4096, 14336), (40, 4096, 4096)],    # the same rows against fewer channels
])
def test_static_scratch_matches_workspace_entry_point(shapes):
    for i, (M, K, N) in enumerate(shapes):   # two calls in a row, the second smaller
        print("static-scratch case", i, (M, K, N), flush=True)
        x, W, s = _case(910 + 17 * i + M, M, K, N)
        ref = msd.msd_gemm_w8a16(x, W, s)
        y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        # the allocator's count of allocation requests (frees by the garbage collector do not move it)
        before = torch.cuda.memory_stats()["allocation.all.allocated"]
        msd.msd_gemm_w8a16_static(x, W, s, y)
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
        torch.cuda.synchronize()
        # same kernels on the same inputs: identical bits
        assert torch.equal(y, ref), (M, K, N)
        yb = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        msd.msd_gemm_w8a16_static(x, W, s, yb)
        torch.cuda.synchronize()
        assert torch.equal(yb, msd.msd_gemm_w8a16(x, W, s, out_dtype=torch.bfloat16))


def test_static_scratch_against_oracle_and_limits():
    import oracle
    M, K, N = 24, 1024, 640
    xb = synth.activations(77, M, K, outliers=True)
    W, s = synth.int8_weights(78, N, K)
    y = torch.empty((M, N), dtype=torch.float32, device="cuda")
    msd.msd_gemm_w8a16_static(bf16_to_dev(xb), to_dev(W), to_dev(s), y)
    torch.cuda.synchronize()
    ref = oracle.gemm_w8a16(xb, W, s)
    err = np.linalg.norm(y.cpu().numpy().astype(np.float64) - ref, axis=1) / np.linalg.norm(ref, axis=1)
    assert err.max() <= 1e-6
    L = msd.lib()
    cap = L.msd_gemm_w8a16_static_scratch_bytes()
    assert cap == (2 << 20) + 4096
    # beyond the built-in buffer: a clear error, nothing enqueued
    p = ctypes.c_void_p(256)
    assert L.msd_gemm_w8a16_static(p, 129, 8192, 8192, p, p, 64, p, 0, 64, None) == -6
    assert L.msd_gemm_w8a16_static(p, 128, 8192, 8192, None, p, 64, p, 0, 64, None) == -1   # fits; null W
    assert L.msd_gemm_w8a16_static(p, 0, 8192, 8192, p, p, 64, p, 0, 64, None) == 0        # empty: no-op
