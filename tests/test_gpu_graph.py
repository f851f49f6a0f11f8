"""The entry points enqueue kernels only (no allocation, no synchronisation, no memset nodes), so a caller may
capture them into a HIP graph.  Each graph is replayed several times with eager work and synchronisations of
the program in between, and every replay is compared with the eager result and, through it, with the oracle."""
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


def _replay_and_check(makers, outs, refs, tol):
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        calls = [mk() for mk in makers]      # a prepared call keeps the stream that was current when it was made
        for c in calls:
            c()
        torch.cuda.synchronize()
        eager = [o.clone() for o in outs]
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for c in calls:
                c()
    for rep in range(3):
        for o in outs:
            o.fill_(float("nan"))            # eager work of the program between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for o, e, r in zip(outs, eager, refs):
            assert torch.equal(o, e), rep
            assert rel_l2(o.float().cpu().numpy(), r) <= tol


def test_gemm_entry_points_in_a_graph(msd):
    calls, outs, refs = [], [], []
    for M, K, N in ((1, 1024, 600), (8, 1024, 600), (32, 1024, 8300), (200, 512, 700)):
        x = synth.activations(M, M, K)
        W, s = synth.int8_weights(M, N, K)
        y = torch.empty((M, N), dtype=torch.float32, device="cuda")
        xd, Wd, sd = bf16_to_dev(x), to_dev(W), to_dev(s)
        calls.append(lambda xd=xd, Wd=Wd, sd=sd, y=y: msd.msd_gemm_w8a16(xd, Wd, sd, y=y, prepare=True))
        outs.append(y)
        refs.append(oracle.gemm_w8a16(x, W, s))
    for M, K, N in ((1, 1024, 300), (20, 1024, 300), (100, 512, 520), (300, 512, 300)):
        x = synth.activations(50 + M, M, K)
        codes, exps = synth.mxfp4_weights(50 + M, N, K)
        y = torch.empty((M, N), dtype=torch.float32, device="cuda")
        xd, cd, ed = bf16_to_dev(x), to_dev(codes), to_dev(exps)
        calls.append(lambda xd=xd, cd=cd, ed=ed, y=y: msd.msd_gemm_w4a16(xd, cd, ed, y=y, prepare=True))
        outs.append(y)
        refs.append(oracle.gemm_w4a16(x, codes, exps))
    _replay_and_check(calls, outs, refs, 2e-6)


def test_attention_and_grouped_gemm_in_a_graph(msd):
    calls, outs, refs = [], [], []
    B, Hq, Hkv, L, d = 2, 8, 2, 2048, 128
    q = synth.queries(3, B, Hq, d)
    Kc, ks, Vc, vs = synth.kv_cache_per_token(3, B, Hkv, L, d)
    o = torch.empty((B, Hq, d), dtype=torch.float32, device="cuda")
    targs = (bf16_to_dev(q), to_dev(Kc), to_dev(Vc), to_dev(ks), to_dev(vs), msd.MSD_PER_TOKEN)
    calls.append(lambda: msd.msd_attn_decode_int8kv(*targs, out=o, prepare=True))
    outs.append(o)
    refs.append(oracle.attn_decode(q, Kc, Vc, ks, vs, oracle.PER_TOKEN))
    E, N, K = 4, 300, 512
    counts = [1, 0, 5, 2]
    x = synth.activations(9, sum(counts), K)
    W = np.stack([synth.int8_weights(9 + e, N, K)[0] for e in range(E)])
    s = np.stack([synth.int8_weights(9 + e, N, K)[1] for e in range(E)])
    offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    y = torch.empty((sum(counts), N), dtype=torch.float32, device="cuda")
    margs = (bf16_to_dev(x), to_dev(offs), to_dev(W), to_dev(s))
    calls.append(lambda: msd.msd_moe_gemm_w8a16(*margs, y=y, prepare=True))
    outs.append(y)
    refs.append(oracle.moe_gemm_w8a16(x, offs, W, s))
    # attention over a latent KV cache: the 16-head layout (query decomposition in the prologue) and the
    # 64-heads-per-workgroup layout (its own decomposition launch), both with split KV and a merge launch
    sm = 1.0 / np.sqrt(192.0)
    for Hl in (16, 40):
        ql = synth.queries(5 + Hl, 1, Hl, 576)
        Cl, sc, _, _ = synth.kv_cache_per_token(5 + Hl, 1, 1, 1500, 576)
        Cl, sc = np.ascontiguousarray(Cl[:, 0]), np.ascontiguousarray(sc[:, 0])
        ol = torch.empty((1, Hl, 512), dtype=torch.float32, device="cuda")
        largs = (bf16_to_dev(ql), to_dev(Cl), to_dev(sc), msd.MSD_PER_TOKEN, sm)
        calls.append(lambda largs=largs, ol=ol: msd.msd_mla_decode_int8kv(*largs, out=ol, prepare=True))
        outs.append(ol)
        refs.append(oracle.mla_decode(ql, Cl, sc, oracle.PER_TOKEN, 512, sm))
    _replay_and_check(calls, outs, refs, 1e-3)
