"""GPU parity: msd_attn_decode_int8kv against the CPU oracle, through the C ABI.

Bar: Q component codes, alpha_Q bits and the two integer score rows S1, S2 bit-exact; the
fp32 output within relative L2 1e-3 of the oracle (P codes are not compared: they depend on
the exp implementation and, for per-token scales, on the tile the scale bound is taken over)
and of the fp64 truth."""
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


CASES = [
    # B, Hq, Hkv, L, mode, kv_len
    (2, 8, 2, 96, "token", None),
    (2, 8, 2, 1000, "token", None),
    (1, 4, 1, 2048, "token", None),          # several KV splits
    (3, 8, 2, 700, "token", [700, 0, 333]),   # ragged lengths incl. an empty entry
    (2, 8, 2, 300, "channel", None),
    (1, 4, 1, 3000, "channel", [2500]),
    (2, 8, 1, 520, "token", None),            # group of 8 query heads per KV head
    (2, 8, 1, 520, "channel", None),
    (2, 3, 3, 130, "token", None),            # no grouping (G = 1)
    (1, 6, 2, 64, "token", None),             # G = 3
    (1, 12, 1, 300, "token", None),           # G = 12: two passes of 8 and 4 heads over the KV range
    (2, 32, 2, 200, "channel", None),         # G = 16
    (1, 40, 2, 130, "channel", None),         # G = 20: ragged last head group
    (1, 48, 1, 1100, "token", [1000]),        # G = 48, several KV splits
]


@pytest.mark.parametrize("B,Hq,Hkv,L,mode,kv_len", CASES)
def test_attn_decode_parity(msd, B, Hq, Hkv, L, mode, kv_len):
    d = 128
    seed = synth.seed_for(4, B * 1000 + L)
    q = synth.queries(seed, B, Hq, d)
    if mode == "token":
        Kc, ks, Vc, vs = synth.kv_cache_per_token(seed, B, Hkv, L, d)
        omode, gmode = oracle.PER_TOKEN, msd.MSD_PER_TOKEN
    else:
        Kc, ks, Vc, vs = synth.kv_cache_per_channel(seed, B, Hkv, L, d)
        omode, gmode = oracle.PER_CHANNEL, msd.MSD_PER_CHANNEL
    kl = None if kv_len is None else np.array(kv_len, np.int32)
    ref, t = oracle.attn_decode(q, Kc, Vc, ks, vs, omode, kv_len=kl, taps=True)
    truth = oracle.truth_attn(q, Kc, Vc, ks, vs, omode, kv_len=kl)
    out, g = msd.msd_attn_decode_int8kv(bf16_to_dev(q), to_dev(Kc), to_dev(Vc), to_dev(ks), to_dev(vs), gmode,
                                        kv_len=None if kl is None else to_dev(kl), taps=True)
    torch.cuda.synchronize()
    lens = [L] * B if kl is None else list(kl)
    live = np.array([l > 0 for l in lens])
    # (the oracle skips entries with no tokens, so their taps are compared for live entries only)
    assert np.array_equal(g["q1"].cpu().numpy()[live], t["q1"][live])
    assert np.array_equal(g["q2"].cpu().numpy()[live], t["q2"][live])
    assert np.array_equal(g["scale"].cpu().numpy().view(np.uint32)[live], t["alpha_q"].view(np.uint32)[live])
    s1, s2 = g["acc1"].cpu().numpy(), g["acc2"].cpu().numpy()
    for b in range(B):
        assert np.array_equal(s1[b, :, :lens[b]], t["s1"][b, :, :lens[b]])
        assert np.array_equal(s2[b, :, :lens[b]], t["s2"][b, :, :lens[b]])
    o = out.cpu().numpy()
    assert np.all(o[~live] == 0)
    assert rel_l2(o[live], ref[live]) <= 1e-3
    assert rel_l2(o[live], truth[live]) <= 1e-3
    # per head, not only in aggregate
    for b in range(B):
        if lens[b] > 0:
            for h in range(Hq):
                assert rel_l2(o[b, h], ref[b, h]) <= 1e-3


def test_attn_bf16_output_and_errors(msd):
    B, Hq, Hkv, L, d = 1, 4, 1, 256, 128
    q = synth.queries(9, B, Hq, d)
    Kc, ks, Vc, vs = synth.kv_cache_per_token(9, B, Hkv, L, d)
    args = (bf16_to_dev(q), to_dev(Kc), to_dev(Vc), to_dev(ks), to_dev(vs), msd.MSD_PER_TOKEN)
    o32 = msd.msd_attn_decode_int8kv(*args)
    o16 = msd.msd_attn_decode_int8kv(*args, out_dtype=torch.bfloat16)
    assert rel_l2(o16.float().cpu().numpy(), o32.cpu().numpy()) < 4e-3
    o32b = msd.msd_attn_decode_int8kv(*args)
    assert torch.equal(o32, o32b)                         # deterministic
    with pytest.raises(msd.MsdError) as e:                # Hq not a multiple of Hkv
        msd.msd_attn_decode_int8kv(torch.zeros((1, 3, 128), dtype=torch.bfloat16, device="cuda"),
                                   torch.zeros((1, 2, 8, 128), dtype=torch.int8, device="cuda"),
                                   torch.zeros((1, 2, 8, 128), dtype=torch.int8, device="cuda"),
                                   torch.ones((1, 2, 8), device="cuda"), torch.ones((1, 2, 8), device="cuda"),
                                   msd.MSD_PER_TOKEN)
    assert e.value.code == -2


def test_attn_extreme_value_scales(msd):
    """Per-token value scales spanning sixty orders of magnitude, a stretch of zero scales and an entry whose
    value scales are all zero: finite outputs that match the oracle and the fp64 truth, zeros for that entry."""
    B, Hq, Hkv, L, d = 3, 8, 2, 1500, 128
    q = synth.queries(41, B, Hq, d)
    Kc, ks, Vc, vs = synth.kv_cache_per_token(41, B, Hkv, L, d)
    vs = vs.copy()
    vs[0, :, :200] = 0.0
    vs[0, :, 200:500] *= 1e-3
    vs[0, :, 500:700] = 1e-35
    vs[0, :, 700:900] *= 1e2
    vs[1, :, :] = np.float32(1e-30) * (1 + np.arange(L, dtype=np.float32) / L)
    vs[1, :, 640:704] *= np.float32(1e25)
    vs[2, :, :] = 0.0
    ref = oracle.attn_decode(q, Kc, Vc, ks, vs, oracle.PER_TOKEN)
    truth = oracle.truth_attn(q, Kc, Vc, ks, vs, oracle.PER_TOKEN)
    out = msd.msd_attn_decode_int8kv(bf16_to_dev(q), to_dev(Kc), to_dev(Vc), to_dev(ks), to_dev(vs), msd.MSD_PER_TOKEN)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert np.all(np.isfinite(o))
    assert np.all(o[2] == 0) and np.all(ref[2] == 0)
    for b in range(2):
        for h in range(Hq):
            assert rel_l2(o[b, h], truth[b, h]) <= 1e-3, (b, h)
            assert rel_l2(o[b, h], ref[b, h]) <= 1e-3, (b, h)
