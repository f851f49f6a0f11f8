"""Pins for the oracle's MSD attention decode step (Sec. 4.2, Alg. 3).

Per-channel scale mode is the paper's statement; per-token mode is this build's reading for
the per-token-per-head KV scales of the measured workload.  Pins: closed-form special cases
(one token; identical keys; identical values), the decomposition bounds applied to P, numpy
integer matmuls on the oracle's own codes, and the fp64 truth."""
import numpy as np
import pytest

import oracle
from paper_2605_13915_amd import synth


def f32(bits):
    return synth.bf16_bits_to_f32(bits).astype(np.float64)


def small_case(seed, mode, B=2, Hq=8, Hkv=2, L=96, d=64):
    q = synth.queries(seed, B, Hq, d)
    if mode == oracle.PER_TOKEN:
        Kc, ks, Vc, vs = synth.kv_cache_per_token(seed, B, Hkv, L, d)
    else:
        Kc, ks, Vc, vs = synth.kv_cache_per_channel(seed, B, Hkv, L, d)
    return q, Kc, Vc, ks, vs


@pytest.mark.parametrize("mode", [oracle.PER_TOKEN, oracle.PER_CHANNEL])
def test_single_token_returns_dequantised_value_row(mode):
    # L = 1: softmax weight is exactly 1 -> P codes (127, 0) -> O = V_real[0] up to fp32 rounding.
    q, Kc, Vc, ks, vs = small_case(51, mode, L=1)
    out = oracle.attn_decode(q, Kc, Vc, ks, vs, mode)
    G = 4
    for b in range(2):
        for h in range(8):
            g = h // G
            vreal = Vc[b, g, 0].astype(np.float64) * (vs[b, g, 0] if mode == oracle.PER_TOKEN else vs[g])
            assert np.allclose(out[b, h], vreal, rtol=3e-7, atol=1e-12)


@pytest.mark.parametrize("mode", [oracle.PER_TOKEN, oracle.PER_CHANNEL])
def test_identical_keys_give_the_mean_value(mode):
    # identical K rows (and identical K scales) -> S constant -> P = 1 everywhere -> O = mean_t V_real[t].
    q, Kc, Vc, ks, vs = small_case(52, mode, L=40)
    Kc[:] = Kc[:, :, :1, :]
    if mode == oracle.PER_TOKEN:
        ks[:] = ks[:, :, :1]
        vs[:] = vs[:, :, :1]        # equal V scales so that P~ = P * const decomposes exactly
    out = oracle.attn_decode(q, Kc, Vc, ks, vs, mode)
    for b in range(2):
        for h in range(8):
            g = h // 4
            sc = vs[b, g, :, None] if mode == oracle.PER_TOKEN else vs[g][None, :]
            mean = (Vc[b, g].astype(np.float64) * sc).mean(axis=0)
            assert np.allclose(out[b, h], mean, rtol=1e-6, atol=1e-9)


@pytest.mark.parametrize("mode", [oracle.PER_TOKEN, oracle.PER_CHANNEL])
def test_identical_values_make_output_independent_of_scores(mode):
    # all V_real rows equal -> O equals that row whatever S is, up to the decomposition error of P.
    q, Kc, Vc, ks, vs = small_case(53, mode, L=200)
    Vc[:] = Vc[:, :, :1, :]
    if mode == oracle.PER_TOKEN:
        vs[:] = vs[:, :, :1]
    out = oracle.attn_decode(q, Kc, Vc, ks, vs, mode)
    for b in range(2):
        for h in range(8):
            g = h // 4
            row = Vc[b, g, 0].astype(np.float64) * (vs[b, g, 0] if mode == oracle.PER_TOKEN else vs[g])
            # sum_t (P_t + err_t) / sum_t P_t with |err_t| <= 1/64516 and sum P >= 1
            assert np.all(np.abs(out[b, h] - row) <= np.abs(row) * 200 / 64516.0 + 1e-9)


@pytest.mark.parametrize("mode", [oracle.PER_TOKEN, oracle.PER_CHANNEL])
def test_taps_invariants_and_integer_products(mode):
    q, Kc, Vc, ks, vs = small_case(54, mode, L=96)
    out, t = oracle.attn_decode(q, Kc, Vc, ks, vs, mode, taps=True)
    B, Hq, d = q.shape
    G = Hq // Kc.shape[1]
    # P in [0,1], max exactly 1, P1 in [0,127], P2 in [-127,127] (Sec. 4.2 step 3)
    assert t["p"].min() >= 0 and np.all(t["p"].max(axis=2) == 1.0)
    assert t["p1"].min() >= 0 and t["p1"].max() <= 127 and np.abs(t["p2"]).max() <= 127
    for b in range(B):
        for h in range(Hq):
            g = h // G
            # S1, S2 are plain integer products of the query codes with the INT8 keys
            assert np.array_equal(t["s1"][b, h].astype(np.int64), Kc[b, g].astype(np.int64) @ t["q1"][b, h].astype(np.int64))
            assert np.array_equal(t["s2"][b, h].astype(np.int64), Kc[b, g].astype(np.int64) @ t["q2"][b, h].astype(np.int64))
            # decomposition error of P (or P*s_V) obeys Thm 1 with M = 1 (or max s_V)
            if mode == oracle.PER_TOKEN:
                top = float(vs[b, g].max())
                pt = t["p"][b, h].astype(np.float64) * vs[b, g].astype(np.float64)
            else:
                top = 1.0
                pt = t["p"][b, h].astype(np.float64)
            rec = top / 127 * t["p1"][b, h] + top / 127 / 254 * t["p2"][b, h]
            assert np.all(np.abs(pt - rec) <= top / 64516.0 * (1 + 1e-4) + pt * 2.0 ** -22)
    # the query decomposition is the INT8 decomposition of Q (per-token) / of Q*s_K (per-channel)
    if mode == oracle.PER_TOKEN:
        q1, q2, al, _ = oracle.decompose_int8(q.reshape(B * Hq, d))
        assert np.array_equal(q1.reshape(B, Hq, d), t["q1"]) and np.array_equal(al.reshape(B, Hq), t["alpha_q"])
    else:
        qt = f32(q) * np.repeat(ks, G, axis=0)[None].astype(np.float64)
        a = t["alpha_q"].astype(np.float64)[..., None]
        assert np.all(np.abs(qt - (a * t["q1"] + a / 254 * t["q2"])) <= np.abs(qt).max(axis=2, keepdims=True) / 64516 * (1 + 1e-3))


@pytest.mark.parametrize("mode", [oracle.PER_TOKEN, oracle.PER_CHANNEL])
def test_against_fp64_truth_and_numpy_softmax(mode):
    q, Kc, Vc, ks, vs = small_case(55, mode, B=2, Hq=8, Hkv=2, L=512, d=128)
    truth = oracle.truth_attn(q, Kc, Vc, ks, vs, mode)
    # the truth itself against a numpy softmax
    G = 4
    for b in range(2):
        for h in range(8):
            g = h // G
            if mode == oracle.PER_TOKEN:
                Kr = Kc[b, g].astype(np.float64) * ks[b, g, :, None]
                Vr = Vc[b, g].astype(np.float64) * vs[b, g, :, None]
            else:
                Kr = Kc[b, g].astype(np.float64) * ks[g][None, :]
                Vr = Vc[b, g].astype(np.float64) * vs[g][None, :]
            s = Kr @ f32(q[b, h]) / np.sqrt(128.0)
            p = np.exp(s - s.max())
            assert np.allclose(truth[b, h], p @ Vr / p.sum(), rtol=1e-10, atol=1e-13)
    out = oracle.attn_decode(q, Kc, Vc, ks, vs, mode)
    rel = np.linalg.norm(out - truth) / np.linalg.norm(truth)
    # far below the 0.49 % the paper's own simulation reports (Sec. 6.4 table); the bound
    # from Thm 1 on Q and P predicts a few 1e-4 here
    assert rel < 1e-3


def test_kv_len_and_gqa_mapping():
    q, Kc, Vc, ks, vs = small_case(56, oracle.PER_TOKEN, L=64)
    kv_len = np.array([64, 17], np.int32)
    out = oracle.attn_decode(q, Kc, Vc, ks, vs, oracle.PER_TOKEN, kv_len=kv_len)
    ref1 = oracle.attn_decode(q[1:], Kc[1:, :, :17].copy(), Vc[1:, :, :17].copy(), ks[1:, :, :17].copy(),
                              vs[1:, :, :17].copy(), oracle.PER_TOKEN)
    assert np.array_equal(out[1], ref1[0])
    # query heads of one group read the same KV head: swapping KV heads changes groups only
    out_sw = oracle.attn_decode(q, Kc[:, ::-1].copy(), Vc[:, ::-1].copy(), ks[:, ::-1].copy(), vs[:, ::-1].copy(),
                                oracle.PER_TOKEN, kv_len=kv_len)
    q_sw = np.concatenate([q[:, 4:], q[:, :4]], axis=1)
    out_ref = oracle.attn_decode(q_sw, Kc, Vc, ks, vs, oracle.PER_TOKEN, kv_len=kv_len)
    assert np.array_equal(out_sw[:, :4], out_ref[:, 4:]) and np.array_equal(out_sw[:, 4:], out_ref[:, :4])


def test_kv_len_outside_the_cache_is_clamped():
    """kv_len above L reads as L (what the library does), negative as empty: no read past the cache
    (this test also runs under AddressSanitizer, test_oracle_sanitized.py)."""
    q, Kc, Vc, ks, vs = small_case(57, oracle.PER_TOKEN, L=48)
    full = oracle.attn_decode(q, Kc, Vc, ks, vs, oracle.PER_TOKEN)
    over = oracle.attn_decode(q, Kc, Vc, ks, vs, oracle.PER_TOKEN, kv_len=np.array([49, 10 ** 6], np.int32))
    assert np.array_equal(over, full)
    neg = oracle.attn_decode(q, Kc, Vc, ks, vs, oracle.PER_TOKEN, kv_len=np.array([-3, 48], np.int32))
    assert np.all(neg[0] == 0) and np.array_equal(neg[1], full[1])
    tr_full = oracle.truth_attn(q, Kc, Vc, ks, vs, oracle.PER_TOKEN)
    tr_over = oracle.truth_attn(q, Kc, Vc, ks, vs, oracle.PER_TOKEN, kv_len=np.array([4096, 48], np.int32))
    assert np.array_equal(tr_over, tr_full)


def test_per_token_mode_reduces_to_the_per_channel_statement_for_uniform_scales():
    """Pin of the per-token reading against the paper's own (per-channel) statement: with every
    per-token scale equal to one power of two c, and every per-channel scale equal to the same c,
    both modes describe the same dequantised K and V, and scaling by a power of two is exact in
    every step -- so the two code paths must produce identical Q, S and P codes and the same
    output up to the one place where they differ in rounding (alpha_P = fl(c/127) against the
    exact constant 1/127)."""
    B, Hq, Hkv, d, L = 2, 8, 2, 128, 300
    rng = np.random.default_rng(5)
    q = synth.queries(11, B, Hq, d)
    Kc = rng.integers(-127, 128, (B, Hkv, L, d), dtype=np.int8)
    Vc = rng.integers(-127, 128, (B, Hkv, L, d), dtype=np.int8)
    for ck, cv in ((2.0 ** -6, 2.0 ** -5), (1.0, 1.0), (2.0 ** -3, 4.0)):
        kt = np.full((B, Hkv, L), ck, np.float32)
        vt = np.full((B, Hkv, L), cv, np.float32)
        kc = np.full((Hkv, d), ck, np.float32)
        vc = np.full((Hkv, d), cv, np.float32)
        o_t, t_t = oracle.attn_decode(q, Kc, Vc, kt, vt, oracle.PER_TOKEN, taps=True)
        o_c, t_c = oracle.attn_decode(q, Kc, Vc, kc, vc, oracle.PER_CHANNEL, taps=True)
        for key in ("q1", "q2", "s1", "s2", "p1", "p2"):
            assert np.array_equal(t_t[key], t_c[key]), key
        assert np.array_equal(t_t["p"], t_c["p"])
        err = np.linalg.norm(o_t.astype(np.float64) - o_c) / np.linalg.norm(o_c)
        assert err < 1e-7


def test_per_token_scales_are_applied_to_their_own_token():
    """Pin of the per-token indexing: multiplying s_K[t] by 2^e_t is the same as multiplying the
    INT8 row K[t] by 2^e_t (small codes, so the product is still INT8) -- exactly, because the
    integer dot products scale by 2^e_t and the merge multiplies by a power of two.  The same
    move on V changes alpha_P (it is max_t s_V[t] / 127), so there the two runs agree within the
    decomposition error only, which still separates a right index from a wrong one by orders of
    magnitude."""
    B, Hq, Hkv, d, L = 2, 8, 2, 128, 300
    rng = np.random.default_rng(7)
    q = synth.queries(13, B, Hq, d)
    Kc = rng.integers(-31, 32, (B, Hkv, L, d), dtype=np.int8)
    Vc = rng.integers(-31, 32, (B, Hkv, L, d), dtype=np.int8)
    e = rng.integers(0, 3, (B, Hkv, L))
    f = rng.integers(0, 3, (B, Hkv, L))
    ck, cv = 2.0 ** -6, 2.0 ** -5
    ku = np.full((B, Hkv, L), ck, np.float32)
    vu = np.full((B, Hkv, L), cv, np.float32)
    ks = (ck * 2.0 ** e).astype(np.float32)
    vs = (cv * 2.0 ** f).astype(np.float32)
    K2 = (Kc.astype(np.int32) * (1 << e)[..., None]).astype(np.int8)
    V2 = (Vc.astype(np.int32) * (1 << f)[..., None]).astype(np.int8)
    o1, t1 = oracle.attn_decode(q, Kc, Vc, ks, vu, oracle.PER_TOKEN, taps=True)
    o2, t2 = oracle.attn_decode(q, K2, Vc, ku, vu, oracle.PER_TOKEN, taps=True)
    assert np.array_equal(o1, o2) and np.array_equal(t1["p"], t2["p"])
    assert np.array_equal(t1["s1"] * (1 << e).repeat(Hq // Hkv, axis=1), t2["s1"])
    o3 = oracle.attn_decode(q, Kc, Vc, ku, vs, oracle.PER_TOKEN)
    o4 = oracle.attn_decode(q, Kc, V2, ku, vu, oracle.PER_TOKEN)
    err = np.linalg.norm(o3.astype(np.float64) - o4) / np.linalg.norm(o4)
    assert err < 2e-4
    # a shifted scale index would be off by O(1)
    o_bad = oracle.attn_decode(q, Kc, Vc, ku, np.roll(vs, 1, axis=2), oracle.PER_TOKEN)
    assert np.linalg.norm(o_bad.astype(np.float64) - o4) / np.linalg.norm(o4) > 0.05


# ------------------------------------------------------------------ latent KV cache (multi-head latent attention)

def latent_case(seed, mode, B=2, Hq=6, L=80, dk=96, dv=64):
    rng = np.random.default_rng(seed)
    q = synth.queries(seed, B, Hq, dk)
    if mode == oracle.PER_TOKEN:
        Cl, sc, _, _ = synth.kv_cache_per_token(seed, B, 1, L, dk)
        Cl, sc = Cl[:, 0], sc[:, 0]
    else:
        Cl, sc, _, _ = synth.kv_cache_per_channel(seed, B, 1, L, dk)
        Cl, sc = Cl[:, 0], sc[0]
    return q, Cl, sc, 1.0 / np.sqrt(48.0 + rng.integers(0, 3))


@pytest.mark.parametrize("mode", [oracle.PER_TOKEN, oracle.PER_CHANNEL])
def test_latent_cache_with_equal_widths_is_alg3_with_one_shared_kv_head(mode):
    # dv = dk and sm_scale = 1/sqrt(dk): the latent form must be bit-identical to the GQA form with Hkv = 1
    # and the cache passed as both K and V
    q, Cl, sc, _ = latent_case(71, mode, dk=64, dv=64)
    out, t = oracle.mla_decode(q, Cl, sc, mode, 64, 1.0 / np.sqrt(64.0), taps=True)
    K4 = Cl[:, None]
    s4 = sc[:, None] if mode == oracle.PER_TOKEN else sc[None]
    ref, tr = oracle.attn_decode(q, K4, K4, s4, s4, mode, taps=True)
    assert np.array_equal(out.view(np.uint32), ref.view(np.uint32))
    for k in ("q1", "q2", "s1", "s2"):
        assert np.array_equal(t[k], tr[k])


@pytest.mark.parametrize("mode", [oracle.PER_TOKEN, oracle.PER_CHANNEL])
def test_latent_cache_scores_use_all_channels_values_the_first_dv(mode):
    q, Cl, sc, sm = latent_case(72, mode)
    B, Hq, dk = q.shape
    dv = 64
    out, t = oracle.mla_decode(q, Cl, sc, mode, dv, sm, taps=True)
    # scores: integer dot products over all dk channels
    for b in range(B):
        assert np.array_equal(t["s1"][b].astype(np.int64), t["q1"][b].astype(np.int64) @ Cl[b].astype(np.int64).T)
        assert np.array_equal(t["s2"][b].astype(np.int64), t["q2"][b].astype(np.int64) @ Cl[b].astype(np.int64).T)
    # values: make the first dv channels of every row equal (the rest stays random): the output is that row,
    # whatever the scores are
    C2 = Cl.copy()
    C2[:, :, :dv] = C2[:, :1, :dv]
    sc2 = sc.copy()
    if mode == oracle.PER_TOKEN:
        sc2[:] = sc2[:, :1]
    out2 = oracle.mla_decode(q, C2, sc2, mode, dv, sm)
    for b in range(B):
        row = C2[b, 0, :dv].astype(np.float64) * (sc2[b, 0] if mode == oracle.PER_TOKEN else sc2[:dv])
        for h in range(Hq):
            assert np.allclose(out2[b, h], row, rtol=2e-4, atol=2e-4 * np.abs(row).max())
    # changing only the channels beyond dv changes the scores but must not enter the values
    C3 = C2.copy()
    C3[:, :, dv:] = -C3[:, :, dv:]
    out3 = oracle.mla_decode(q, C3, sc2, mode, dv, sm)
    for b in range(B):
        row = C2[b, 0, :dv].astype(np.float64) * (sc2[b, 0] if mode == oracle.PER_TOKEN else sc2[:dv])
        assert np.allclose(out3[b], row[None], rtol=2e-4, atol=2e-4 * np.abs(row).max())


@pytest.mark.parametrize("mode", [oracle.PER_TOKEN, oracle.PER_CHANNEL])
def test_latent_cache_against_numpy_softmax_and_fp64_truth(mode):
    q, Cl, sc, sm = latent_case(73, mode, L=200)
    B, Hq, dk = q.shape
    dv = 64
    kv_len = np.array([200, 131], np.int32)
    truth = oracle.truth_mla(q, Cl, sc, mode, dv, sm, kv_len=kv_len)
    qf = f32(q)
    for b in range(B):
        n = int(kv_len[b])
        Kr = Cl[b, :n].astype(np.float64) * (sc[b, :n, None] if mode == oracle.PER_TOKEN else sc[None, :])
        S = qf[b] @ Kr.T * sm
        P = np.exp(S - S.max(axis=1, keepdims=True))
        ref = (P / P.sum(axis=1, keepdims=True)) @ Kr[:, :dv]
        assert np.allclose(truth[b], ref, rtol=1e-10, atol=1e-12)
    out = oracle.mla_decode(q, Cl, sc, mode, dv, sm, kv_len=kv_len)
    num = np.linalg.norm(out - truth)
    assert num / np.linalg.norm(truth) < 1e-3


# ---------------------------------------------------------------- low-precision variant (Sec. 4.4, optimisation opportunities)
def _lowprec_case(seed, mode, L=200, B=2, Hq=8, Hkv=2):
    q, Kc, Vc, ks, vs = small_case(seed, mode, L=L, B=B, Hq=Hq, Hkv=Hkv)
    out, t = oracle.attn_decode(q, Kc, Vc, ks, vs, mode, taps=True, lowprec=True)
    return (q, Kc, Vc, ks, vs), out, t


@pytest.mark.parametrize("mode", [oracle.PER_CHANNEL, oracle.PER_TOKEN])
def test_lowprec_p_codes_equal_an_independent_float16_implementation(mode):
    """The FP16 steps written a second time with numpy's float16 type (correctly rounded +, -, *):
    q1 = rne(v_h), r = v_h - q1, q2 = rne(254 r) (the product taken exactly, as the fused operation does),
    from the oracle's own P row.  Bit for bit."""
    (q, Kc, Vc, ks, vs), out, t = _lowprec_case(71, mode)
    B, Hq, L = t["p"].shape
    G = Hq // Kc.shape[1]
    for b in range(B):
        for h in range(Hq):
            P = t["p"][b, h]
            if mode == oracle.PER_TOKEN:
                sv = vs[b, h // G]
                v = (P * sv).astype(np.float32) * (np.float32(127.0) / sv.max())
            else:
                v = np.float32(127.0) * P
            vh = v.astype(np.float32).astype(np.float16)
            c1 = np.rint(vh.astype(np.float64))                       # round-half-even of an FP16 value, exact
            r = (vh - c1.astype(np.float16)).astype(np.float16)
            assert np.array_equal(r.astype(np.float64), vh.astype(np.float64) - c1)   # the residual is exact
            c2 = np.rint(r.astype(np.float64) * 254.0)                # exact product, round-half-even
            assert np.array_equal(t["p1"][b, h], c1.astype(np.int8)), (b, h)
            assert np.array_equal(t["p2"][b, h], c2.astype(np.int8)), (b, h)
            assert c1.min() >= 0 and c1.max() <= 127 and np.abs(c2).max() <= 127


def test_lowprec_decomposition_bound_and_closed_forms():
    """|v - (q1 + q2/254)| <= 2^-11 v + 1/508 in units of alpha_P (derived in the oracle's header),
    and it is attained to within a factor of two (the bound is not slack by an order of magnitude)."""
    (q, Kc, Vc, ks, vs), out, t = _lowprec_case(72, oracle.PER_CHANNEL, L=4000, B=1, Hq=4, Hkv=1)
    v = 127.0 * t["p"].astype(np.float64)
    rec = t["p1"].astype(np.float64) + t["p2"].astype(np.float64) / 254.0
    err = np.abs(v - rec)
    bound = 2.0 ** -11 * v + 1.0 / 508.0
    assert np.all(err <= bound * (1 + 1e-6) + 127.0 * 2.0 ** -24)
    assert (err / bound).max() > 0.5
    # the largest probability of every row is exp(0) = 1: codes (127, 0), reconstructed exactly
    imax = t["p"].argmax(axis=2)
    for h in range(4):
        assert t["p"][0, h, imax[0, h]] == 1.0
        assert t["p1"][0, h, imax[0, h]] == 127 and t["p2"][0, h, imax[0, h]] == 0


def test_lowprec_half_probability_ties_to_even():
    """Two identical keys with scores S and S - ln 2 are not constructible exactly; instead feed the FP16 steps
    through a row where P is exactly 1/2: L = 2 identical keys give P = (1, 1); scaled value scales make
    P~ = (s, s/2).  127 * 1/2 = 63.5 is an exact tie: q1 = 64 (even), r = -1/2, q2 = -127, reconstruction exact."""
    B, Hq, Hkv, d, L = 1, 1, 1, 128, 2
    rng = np.random.default_rng(5)
    q = synth.queries(5, B, Hq, d)
    Kc = np.repeat(rng.integers(-127, 128, (B, Hkv, 1, d), dtype=np.int8), L, axis=2)
    Vc = rng.integers(-127, 128, (B, Hkv, L, d), dtype=np.int8)
    ks = np.ones((B, Hkv, L), np.float32)
    vs = np.array([[[0.25, 0.125]]], np.float32)
    out, t = oracle.attn_decode(q, Kc, Vc, ks, vs, oracle.PER_TOKEN, taps=True, lowprec=True)
    assert np.array_equal(t["p"][0, 0], [1.0, 1.0])
    assert list(t["p1"][0, 0]) == [127, 64] and list(t["p2"][0, 0]) == [0, -127]
    ref = (0.25 * Vc[0, 0, 0].astype(np.float64) + 0.125 * Vc[0, 0, 1].astype(np.float64)) / 2.0
    assert np.allclose(out[0, 0], ref, rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("mode", [oracle.PER_CHANNEL, oracle.PER_TOKEN])
def test_lowprec_integer_merge_and_accuracy_ordering(mode):
    """The integer S merge changes nothing that is defined exactly: Q codes, S1, S2 equal the main variant's,
    P differs by fp32 roundings only.  Accuracy against the fp64 truth: still well below 1e-3, and worse than
    the fp32 arithmetic (the FP16 rounding of the large probabilities), as the bound says."""
    (q, Kc, Vc, ks, vs), out, t = _lowprec_case(73, mode, L=700)
    main, tm = oracle.attn_decode(q, Kc, Vc, ks, vs, mode, taps=True)
    for k in ("q1", "q2", "s1", "s2"):
        assert np.array_equal(t[k], tm[k])
    assert np.allclose(t["p"], tm["p"], rtol=2e-5, atol=1e-9)
    truth = oracle.truth_attn(q, Kc, Vc, ks, vs, mode)
    e_low = np.linalg.norm(out - truth) / np.linalg.norm(truth)
    e_main = np.linalg.norm(main - truth) / np.linalg.norm(truth)
    assert e_low < 1e-3
    assert e_main < e_low < 8 * e_main + 1e-5
