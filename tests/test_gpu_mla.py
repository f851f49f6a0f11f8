"""GPU parity: msd_mla_decode_int8kv (attention over a latent KV cache, 576-channel keys / 512-channel
values from the same cached rows) against the CPU oracle, through the C ABI.  Bar as for the grouped-query
kernel: Q codes, alpha_Q and both integer score rows bit-exact, outputs within relative L2 1e-3 of the
oracle and of the fp64 truth, per head."""
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


def _case(seed, mode, B, Hq, L, ld=576):
    q = synth.queries(seed, B, Hq, 576)
    if mode == "token":
        Cl, sc, _, _ = synth.kv_cache_per_token(seed, B, 1, L, ld)
        return q, np.ascontiguousarray(Cl[:, 0]), np.ascontiguousarray(sc[:, 0])
    Cl, sc, _, _ = synth.kv_cache_per_channel(seed, B, 1, L, ld)
    return q, np.ascontiguousarray(Cl[:, 0]), np.ascontiguousarray(sc[0, :576])


CASES = [
    # B, Hq, L, mode, kv_len, ld
    (2, 8, 96, "token", None, 576),
    (1, 16, 700, "token", None, 576),          # two token streams, ragged last tile
    (3, 5, 300, "token", [300, 0, 77], 576),   # ragged lengths incl. an empty entry, partial head group
    (2, 8, 260, "channel", None, 576),
    (1, 16, 2300, "token", [2070], 576),       # several KV splits; the last split leaves one stream without a tile
    (1, 20, 2048, "channel", [1900], 576),     # 32-head layout, partly filled; several KV splits
    (2, 32, 333, "token", None, 576),          # 32-head layout, full
    (2, 4, 130, "token", None, 640),           # padded cache rows (ld > 576)
    (1, 40, 450, "channel", None, 576),        # 64-head layout, partly filled
    (1, 72, 200, "token", [131], 576),         # two head blocks, the second partly filled
    (1, 128, 520, "token", None, 576),         # 128 heads on one latent: two head blocks of 64
]


@pytest.mark.parametrize("B,Hq,L,mode,kv_len,ld", CASES)
def test_mla_decode_parity(msd, B, Hq, L, mode, kv_len, ld):
    q, Cl, sc = _case(synth.seed_for(9, B * 1000 + L + Hq), mode, B, Hq, L, ld)
    omode, gmode = (oracle.PER_TOKEN, msd.MSD_PER_TOKEN) if mode == "token" else (oracle.PER_CHANNEL, msd.MSD_PER_CHANNEL)
    sm = 1.0 / np.sqrt(192.0)
    kl = None if kv_len is None else np.array(kv_len, np.int32)
    ref, t = oracle.mla_decode(q, Cl, sc, omode, 512, sm, kv_len=kl, taps=True)
    truth = oracle.truth_mla(q, Cl, sc, omode, 512, sm, kv_len=kl)
    out, g = msd.msd_mla_decode_int8kv(bf16_to_dev(q), to_dev(Cl), to_dev(sc), gmode, sm,
                                       kv_len=None if kl is None else to_dev(kl), taps=True)
    torch.cuda.synchronize()
    lens = [L] * B if kl is None else list(kl)
    live = np.array([l > 0 for l in lens])
    assert np.array_equal(g["q1"].cpu().numpy()[live], t["q1"][live])
    assert np.array_equal(g["q2"].cpu().numpy()[live], t["q2"][live])
    assert np.array_equal(g["scale"].cpu().numpy().view(np.uint32)[live], t["alpha_q"].view(np.uint32)[live])
    s1, s2 = g["acc1"].cpu().numpy(), g["acc2"].cpu().numpy()
    for b in range(B):
        assert np.array_equal(s1[b, :, :lens[b]], t["s1"][b, :, :lens[b]])
        assert np.array_equal(s2[b, :, :lens[b]], t["s2"][b, :, :lens[b]])
    o = out.cpu().numpy()
    assert np.all(np.isfinite(o)) and np.all(o[~live] == 0)
    for b in range(B):
        if lens[b] > 0:
            for h in range(Hq):
                assert rel_l2(o[b, h], ref[b, h]) <= 1e-3, (b, h)
                assert rel_l2(o[b, h], truth[b, h]) <= 1e-3, (b, h)


def test_mla_bf16_output_and_errors(msd):
    q, Cl, sc = _case(5, "token", 1, 8, 256)
    sm = 1.0 / np.sqrt(192.0)
    ref = oracle.mla_decode(q, Cl, sc, oracle.PER_TOKEN, 512, sm)
    ob = msd.msd_mla_decode_int8kv(bf16_to_dev(q), to_dev(Cl), to_dev(sc), msd.MSD_PER_TOKEN, sm,
                                   out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert rel_l2(ob.float().cpu().numpy(), ref) <= 1e-2
    with pytest.raises(msd.MsdError) as e:       # keys must be 576 wide
        msd.msd_mla_decode_int8kv(bf16_to_dev(q[:, :, :512].copy()), to_dev(Cl), to_dev(sc), msd.MSD_PER_TOKEN, sm)
    assert e.value.code == -2
    tiny = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(msd.MsdError) as e:
        msd.msd_mla_decode_int8kv(bf16_to_dev(q), to_dev(Cl), to_dev(sc), msd.MSD_PER_TOKEN, sm, ws=tiny)
    assert e.value.code == -3


def _random_cases(n, seed=77):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        B = int(rng.integers(1, 5))
        Hq = int(rng.choice([1, 2, 7, 8, 9, 15, 16, 17, 31, 32, 33, 50, 64, 65, 100, 130]))
        L = int(rng.choice([1, 5, 63, 64, 65, 127, 128, 129, 255, 256, 257, 500, 511, 513, 1000, 1500, 2100, 3000]))
        mode = "token" if rng.integers(0, 2) else "channel"
        ld = int(rng.choice([576, 592, 640]))
        ragged = bool(rng.integers(0, 2))
        out.append((B, Hq, L, mode, ld, ragged, 1000 + i))
    return out


@pytest.mark.parametrize("B,Hq,L,mode,ld,ragged,seed", _random_cases(24))
def test_mla_decode_random_shapes(msd, B, Hq, L, mode, ld, ragged, seed):
    """Seeded random shapes across the three wave layouts, the head-block and KV-split boundaries, ragged
    lengths and padded rows: outputs within 1e-3 of the oracle per head, zeros for empty entries."""
    q, Cl, sc = _case(seed, mode, B, Hq, L, ld)
    omode, gmode = (oracle.PER_TOKEN, msd.MSD_PER_TOKEN) if mode == "token" else (oracle.PER_CHANNEL, msd.MSD_PER_CHANNEL)
    sm = 1.0 / np.sqrt(192.0)
    kl = None
    if ragged:
        kl = np.random.default_rng(seed).integers(0, L + 1, size=B).astype(np.int32)
    ref = oracle.mla_decode(q, Cl, sc, omode, 512, sm, kv_len=kl)
    out = msd.msd_mla_decode_int8kv(bf16_to_dev(q), to_dev(Cl), to_dev(sc), gmode, sm,
                                    kv_len=None if kl is None else to_dev(kl))
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert np.all(np.isfinite(o))
    lens = [L] * B if kl is None else list(kl)
    for b in range(B):
        if lens[b] == 0:
            assert np.all(o[b] == 0)
            continue
        for h in range(Hq):
            assert rel_l2(o[b, h], ref[b, h]) <= 1e-3, (b, h)


def test_mla_extreme_token_scales(msd):
    """Per-token scales spanning sixty orders of magnitude inside one KV split, a stretch of zero scales at the
    start and an entry whose scales are all zero: outputs stay finite, match the oracle and the fp64 truth,
    and the all-zero entry gives zeros."""
    B, Hq, L = 3, 16, 1400
    q, Cl, sc = _case(31, "token", B, Hq, L)
    sc = sc.copy()
    sc[0, :200] = 0.0
    sc[0, 200:500] *= 1e-3
    sc[0, 500:700] = 1e-35
    sc[0, 700:900] *= 1e2
    sc[0, 900:] *= 1e-4
    sc[1, :] = np.float32(1e-30) * (1 + np.arange(L, dtype=np.float32) / L)
    sc[1, 640:704] *= np.float32(1e25)
    sc[2, :] = 0.0
    sm = 1.0 / np.sqrt(192.0)
    ref = oracle.mla_decode(q, Cl, sc, oracle.PER_TOKEN, 512, sm)
    truth = oracle.truth_mla(q, Cl, sc, oracle.PER_TOKEN, 512, sm)
    out = msd.msd_mla_decode_int8kv(bf16_to_dev(q), to_dev(Cl), to_dev(sc), msd.MSD_PER_TOKEN, sm)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert np.all(np.isfinite(o))
    assert np.all(o[2] == 0) and np.all(ref[2] == 0)
    for b in range(2):
        for h in range(Hq):
            assert rel_l2(o[b, h], truth[b, h]) <= 1e-3, (b, h)
            assert rel_l2(o[b, h], ref[b, h]) <= 1e-3, (b, h)
