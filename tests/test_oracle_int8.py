"""Pins for the oracle's two-pass INT8 decomposition and W8A16 GEMM (Sec. 3.2, Alg. 1).

Nothing here re-types the oracle's formula: the checks are the paper's theorem, closed
forms that follow from it, hand-worked special cases, brute force and numpy's own integer
matmul / fp64 arithmetic.
"""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2605_13915_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def f32(bits):
    return synth.bf16_bits_to_f32(bits).astype(np.float64)


def make_rows(seed, M, K, dist="normal", outliers=True, scale=1.0):
    return synth.activations(seed, M, K, outliers=outliers, dist=dist, scale=scale)


@pytest.mark.parametrize("dist,outliers,scale", [("normal", True, 1.0), ("normal", False, 1e-3),
                                                 ("uniform", False, 7.0), ("laplace", True, 100.0)])
def test_theorem1_bound_and_pass1_residual(dist, outliers, scale):
    # Thm 1 (Sec. 5.1): |x - (a q1 + b q2)| <= M/64516; its proof: |x - a q1| <= a/2.
    x = make_rows(11, 16, 2048, dist, outliers, scale)
    q1, q2, al, be = oracle.decompose_int8(x)
    xf = f32(x)
    a = al.astype(np.float64)[:, None]
    b = be.astype(np.float64)[:, None]
    M = np.abs(xf).max(axis=1, keepdims=True)
    rec = a * q1 + b * q2
    assert np.all(np.abs(xf - rec) <= M / 64516.0 * (1 + 2.0 ** -16))
    # (slack: x/alpha is an fp32 quotient, so a value within 127*2^-24 of a tie may round across it)
    assert np.all(np.abs(xf - a * q1) <= a / 2 * (1 + 2.0 ** -15))
    # the bound is close to tight on 32k samples
    assert (np.abs(xf - rec) / (M / 64516.0)).max() > 0.97
    # zero clipping: both code vectors stay inside [-127, 127] (Sec. 7.2)
    assert q1.min() >= -127 and q1.max() <= 127 and q2.min() >= -127 and q2.max() <= 127


def test_scales_are_the_papers_quotients():
    # alpha = ||x||_inf / 127 and beta = alpha / 254 as correctly rounded fp32 quotients,
    # checked with exact rational arithmetic.
    x = make_rows(12, 8, 512)
    _, _, al, be = oracle.decompose_int8(x)
    xf = f32(x)
    for m in range(8):
        M = Fraction(float(np.abs(xf[m]).max()))
        exact_a = M / 127
        a = Fraction(float(al[m]))
        ulp = Fraction(float(np.spacing(al[m])))
        assert abs(a - exact_a) <= ulp / 2
        exact_b = a / 254
        ulpb = Fraction(float(np.spacing(be[m])))
        assert abs(Fraction(float(be[m])) - exact_b) <= ulpb / 2


def test_base254_fixed_point_closed_form():
    # With beta = alpha/254 the pair (q1, q2) is the base-254 digit expansion of the
    # 16-bit fixed-point code z = round(x/beta): |x/beta - (254 q1 + q2)| <= 1/2 (+ fp32 slack).
    x = make_rows(13, 8, 4096)
    q1, q2, al, be = oracle.decompose_int8(x)
    xf = f32(x)
    z = 254.0 * q1 + q2
    t = xf / be.astype(np.float64)[:, None]
    assert np.all(np.abs(t - z) <= 0.5 + 1e-2)
    assert np.abs(z).max() <= 127 * 254 + 127


def test_extremal_element_maps_to_127_and_zero():
    # The element attaining the row max satisfies x/alpha = 127 exactly-rounded, so q1 = +-127
    # and its residual code is 0 (Sec. 3.3, "the extremal element ... rounding error is zero").
    x = make_rows(14, 32, 1024)
    q1, q2, _, _ = oracle.decompose_int8(x)
    xf = f32(x)
    j = np.abs(xf).argmax(axis=1)
    r = np.arange(32)
    assert np.all(q1[r, j] == 127 * np.sign(xf[r, j]))
    assert np.all(np.abs(q2[r, j]) <= 1)


def test_hand_worked_row_with_ties():
    # Hand-worked: x = [127, 64, -1, 0.5, -0.5, 1.5, 2.5, 0]; M = 127, alpha = 1, beta = fp32(1/254).
    # Ties go to even: 0.5 -> 0, -0.5 -> 0, 1.5 -> 2, 2.5 -> 2.  Residuals +-0.5 -> q2 = +-127.
    vals = np.array([[127.0, 64.0, -1.0, 0.5, -0.5, 1.5, 2.5, 0.0]], np.float32)
    x = synth.f32_to_bf16_bits(vals)
    q1, q2, al, be = oracle.decompose_int8(x)
    assert al[0] == np.float32(1.0)
    assert be[0] == np.float32(1.0) / np.float32(254.0)
    assert q1[0].tolist() == [127, 64, -1, 0, 0, 2, 2, 0]
    assert q2[0].tolist() == [0, 0, 0, 127, -127, -127, 127, 0]


def test_zero_row_and_single_element():
    x = np.zeros((2, 64), np.uint16)
    x[1, 5] = synth.f32_to_bf16_bits(np.array([-3.0], np.float32))[0]
    q1, q2, al, be = oracle.decompose_int8(x)
    assert al[0] == 0 and be[0] == 0 and not q1[0].any() and not q2[0].any()
    assert q1[1, 5] == -127 and q2[1, 5] == 0 and np.count_nonzero(q1[1]) == 1


def test_brute_force_tiny_rows():
    # Exhaustive search over all (q1, q2) in [-127,127]^2: no pair beats the greedy error by
    # more than fp32 slack, and for the greedy q1 the greedy q2 is the exhaustive minimiser.
    x = make_rows(15, 3, 8, outliers=False)
    q1, q2, al, be = oracle.decompose_int8(x)
    xf = f32(x)
    grid = np.arange(-127, 128, dtype=np.float64)
    for m in range(3):
        a, b = float(al[m]), float(be[m])
        for k in range(8):
            err = np.abs(xf[m, k] - (a * grid[:, None] + b * grid[None, :]))
            greedy = abs(xf[m, k] - (a * q1[m, k] + b * q2[m, k]))
            assert greedy <= b / 2 * (1 + 1e-5)
            assert err.min() <= greedy + 1e-300
            row = err[int(q1[m, k]) + 127]
            assert abs(row.min() - greedy) <= b * 1e-6
            assert np.argmin(row) - 127 == q2[m, k] or abs(row[np.argmin(row)] - greedy) <= b * 1e-6


def test_fractional_scaling_variant_bound():
    # Sec. 3.3: alpha = M/127.49, beta = alpha/254.98 tightens the bound to ~M/65015.
    x = make_rows(16, 16, 2048)
    q1, q2, al, be = oracle.decompose_int8(x, fractional=True)
    xf = f32(x)
    M = np.abs(xf).max(axis=1, keepdims=True)
    rec = al.astype(np.float64)[:, None] * q1 + be.astype(np.float64)[:, None] * q2
    bound = M / (127.49 * 254.98 * 2)
    assert np.all(np.abs(xf - rec) <= bound * (1 + 1e-4))
    assert abs(127.49 * 254.98 * 2 - 65015) < 1.0          # the constant the paper prints
    assert np.abs(q1).max() <= 127 and np.abs(q2).max() <= 127


# ---------------------------------------------------------------- GEMM (Alg. 1)

def test_gemm_integer_partials_match_numpy_int64():
    x = make_rows(21, 5, 192)
    W, s = synth.int8_weights(21, 37, 192)
    y, t = oracle.gemm_w8a16(x, W, s, taps=True)
    assert not t["overflow"]
    assert np.array_equal(t["acc1"].astype(np.int64), t["q1"].astype(np.int64) @ W.astype(np.int64).T)
    assert np.array_equal(t["acc2"].astype(np.int64), t["q2"].astype(np.int64) @ W.astype(np.int64).T)
    q1, q2, al, be = oracle.decompose_int8(x)
    assert np.array_equal(q1, t["q1"]) and np.array_equal(q2, t["q2"]) and np.array_equal(al, t["alpha"])


def test_gemm_exact_rational_tiny():
    # y = s_W * (alpha*acc1 + beta*acc2) evaluated in exact rationals from the codes.
    x = make_rows(22, 3, 8, outliers=False)
    W, s = synth.int8_weights(22, 4, 8)
    y, t = oracle.gemm_w8a16(x, W, s, taps=True)
    for m in range(3):
        for n in range(4):
            a1 = sum(int(t["q1"][m, k]) * int(W[n, k]) for k in range(8))
            a2 = sum(int(t["q2"][m, k]) * int(W[n, k]) for k in range(8))
            ex = Fraction(float(s[n])) * (Fraction(float(t["alpha"][m])) * a1 + Fraction(float(t["beta"][m])) * a2)
            assert abs(Fraction(float(y[m, n])) - ex) <= abs(ex) * Fraction(1, 2 ** 22) + Fraction(1, 10 ** 30)


def test_gemm_output_bound_against_fp64_truth():
    # Propagating Thm 1 through the dot product:
    # |y_msd - y_true| <= s_W[n] * ||W[n,:]||_1 * M_m / 64516 (+ fp32 output rounding).
    x = make_rows(23, 6, 1024)
    W, s = synth.int8_weights(23, 96, 1024)
    y = oracle.gemm_w8a16(x, W, s).astype(np.float64)
    xf = f32(x)
    truth_np = (xf @ W.astype(np.float64).T) * s.astype(np.float64)[None, :]
    truth = oracle.truth_gemm_w8(x, W, s)
    assert np.allclose(truth, truth_np, rtol=1e-12, atol=1e-12)
    M = np.abs(xf).max(axis=1)
    bound = s.astype(np.float64)[None, :] * np.abs(W.astype(np.float64)).sum(axis=1)[None, :] * M[:, None] / 64516.0
    assert np.all(np.abs(y - truth) <= bound * (1 + 1e-4) + np.abs(truth) * 2.0 ** -23)


def test_gemm_fractional_variant_uses_its_own_constants_throughout():
    # Sec. 3.3: the variant changes the decomposition AND the beta of the merge.  Codes and partial
    # products must be those of the fractional decomposition, the output the exact rational merge with
    # beta = alpha / 254.98f, and the output-level bound tightens to M/65015.
    x = make_rows(27, 5, 256)
    W, s = synth.int8_weights(27, 24, 256)
    y, t = oracle.gemm_w8a16(x, W, s, fractional=True, taps=True)
    q1, q2, al, be = oracle.decompose_int8(x, fractional=True)
    assert np.array_equal(t["q1"], q1) and np.array_equal(t["q2"], q2)
    assert np.array_equal(t["alpha"], al) and np.array_equal(t["beta"], be)
    assert np.array_equal(be, (al / np.float32(254.98)).astype(np.float32))
    assert np.array_equal(t["acc1"].astype(np.int64), q1.astype(np.int64) @ W.astype(np.int64).T)
    assert np.array_equal(t["acc2"].astype(np.int64), q2.astype(np.int64) @ W.astype(np.int64).T)
    for m in range(5):
        for n in range(0, 24, 5):
            ex = Fraction(float(s[n])) * (Fraction(float(al[m])) * int(t["acc1"][m, n]) +
                                          Fraction(float(be[m])) * int(t["acc2"][m, n]))
            assert abs(Fraction(float(y[m, n])) - ex) <= abs(ex) * Fraction(1, 2 ** 22) + Fraction(1, 10 ** 30)
    xf = f32(x)
    truth = oracle.truth_gemm_w8(x, W, s)
    M = np.abs(xf).max(axis=1)
    bound = s.astype(np.float64)[None, :] * np.abs(W.astype(np.float64)).sum(axis=1)[None, :] * M[:, None] / 65015.0
    assert np.all(np.abs(y - truth) <= bound * (1 + 1e-4) + np.abs(truth) * 2.0 ** -23)
    y_main = oracle.gemm_w8a16(x, W, s)
    assert not np.array_equal(y, y_main)          # a different quantiser, not a relabelling


def test_gemv_m1_identity_weights():
    # M = 1 with W = 127 * I and s_W = 1/127 must give back alpha*q1 + beta*q2 per element.
    K = 64
    x = make_rows(24, 1, K, outliers=False)
    W = (np.eye(K, dtype=np.int8) * 127).astype(np.int8)
    s = np.full(K, 1.0 / 127.0, np.float32)
    y, t = oracle.gemm_w8a16(x, W, s, taps=True)
    rec = (t["alpha"].astype(np.float64)[:, None] * t["q1"] + t["beta"].astype(np.float64)[:, None] * t["q2"])
    assert np.allclose(y, rec * 127.0 * float(s[0]), rtol=3e-7, atol=0)
    assert np.allclose(y, f32(x), rtol=0, atol=np.abs(f32(x)).max() / 64000.0)


def test_loose_pins_from_the_papers_tables():
    # Table "error-vs-size" (Sec. 6.2.2): 1024x1024, small batch, Gaussian activation, s_W ~ U[0.01,1]:
    # MSD 0.004 % rel. L2, about 200x below the BF16 dequant baseline.  Seeds are unknown, so
    # only the order of magnitude and the ratio are pinned.
    with open(os.path.join(GOLDEN, "paper_tables.json")) as f:
        gold = json.load(f)["error_vs_size"]["1024"]
    rng = np.random.default_rng(5)
    K = N = 1024
    x = synth.f32_to_bf16_bits(rng.standard_normal((4, K), dtype=np.float32))
    W = rng.integers(-127, 128, size=(N, K), dtype=np.int8)
    s = rng.uniform(0.01, 1.0, N).astype(np.float32)
    truth = oracle.truth_gemm_w8(x, W, s)
    msd = oracle.gemm_w8a16(x, W, s)
    deq = oracle.dequant_gemm_w8a16(x, W, s)
    e_msd = np.linalg.norm(msd - truth) / np.linalg.norm(truth)
    e_deq = np.linalg.norm(deq - truth) / np.linalg.norm(truth)
    assert gold["msd_rel_l2"] / 4 < e_msd < gold["msd_rel_l2"] * 2.5
    assert e_deq / e_msd > 30


# ---------------------------------------------------------------- grouped GEMM (Sec. 7.5)

def test_moe_grouped_gemm_is_alg1_per_row_with_its_experts_weights():
    # every output row depends on its own activation row and on its expert's weights only: it must equal
    # the M = 1 product of that row, whatever the other rows and the grouping are; experts without rows
    # contribute nothing; negating an expert's weights negates exactly its rows.
    E, N, K, T = 5, 24, 128, 11
    x = make_rows(31, T, K)
    W = np.stack([synth.int8_weights(31 + e, N, K)[0] for e in range(E)])
    s = np.stack([synth.int8_weights(31 + e, N, K)[1] for e in range(E)])
    offs = np.array([0, 3, 3, 4, 10, 11])            # expert 1 is empty
    y = oracle.moe_gemm_w8a16(x, offs, W, s)
    owner = np.searchsorted(offs, np.arange(T), side="right") - 1
    assert list(owner) == [0, 0, 0, 2, 3, 3, 3, 3, 3, 3, 4]
    for t in range(T):
        assert np.array_equal(y[t:t + 1], oracle.gemm_w8a16(x[t:t + 1], W[owner[t]], s[owner[t]]))
    W2 = W.copy()
    W2[3] = -W2[3]
    y2 = oracle.moe_gemm_w8a16(x, offs, W2, s)
    assert np.array_equal(y2[4:10], -y[4:10]) and np.array_equal(y2[:4], y[:4]) and np.array_equal(y2[10:], y[10:])
    # rows not assigned to any expert stay zero
    y3 = oracle.moe_gemm_w8a16(x, np.array([0, 3, 3, 4, 8, 9]), W, s)
    assert np.all(y3[9:] == 0) and np.array_equal(y3[:8], y[:8])


def test_maximum_k_extremal_row_stays_inside_int32():
    # K = 131072 is the largest contraction length the ABI accepts: with every code at +-127 on both sides
    # the partial product is 127 * 127 * K = 2 114 060 288 < 2^31 (closed form), one more 16-element chunk of
    # such codes would still fit, twice the length would not.
    K = 131072
    x = np.full((1, K), synth.f32_to_bf16_bits(np.array([3.0], np.float32))[0], np.uint16)
    W = np.full((2, K), 127, np.int8)
    W[1] = -127
    s = np.array([1.0, 1.0], np.float32)
    y, t = oracle.gemm_w8a16(x, W, s, taps=True)
    assert not t["overflow"]
    assert np.all(t["q1"] == 127) and np.all(t["q2"] == 0)
    assert t["acc1"][0, 0] == 127 * 127 * K == 2114060288 and t["acc1"][0, 1] == -2114060288
    assert 127 * 127 * K < 2 ** 31 <= 127 * 127 * 2 * K
    assert abs(float(y[0, 0]) - 3.0 * 127 * K) <= 3.0 * 127 * K * 2.0 ** -22
