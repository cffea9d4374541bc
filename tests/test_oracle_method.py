"""Pins for the method-level pieces of the oracle: Lemma 3.1 (exponent add == multiply by
2^n), Algorithm 1's chunk invariance, Eq. (4) == Eq. (2), the r_i range, the FP32 overflow
remark, and the FLOP / byte accounting against Tables 2 and 5."""
import math
import os

import numpy as np
import pytest

from oracle import amla_oracle as orc
from paper_2509_25224_amd import accounting as acc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


# ----------------------------------------------------------------------------- Lemma 3.1
def test_worked_example_bits():
    (pattern, fval, e), = _rows("example_3_1.txt")
    i = int(pattern, 2)
    assert i == int(e) * 2 ** 23
    assert float(orc.as_fp32(np.int32(i))) == float(fval)
    assert int(orc.as_int32(np.float32(fval))) == i
    # adding 1 * 2^23 doubles it
    assert float(orc.exponent_add(np.float32(fval), 1)) == 1.0


def test_lemma_bit_exact_against_ldexp_all_exponents():
    rng = np.random.default_rng(1)
    mant = np.concatenate([[0, 1, 2 ** 22, 2 ** 23 - 1], rng.integers(0, 2 ** 23, 60)]).astype(np.int64)
    for E in range(1, 255):
        for sign in (0, 1):
            I = (sign << 31) | (E << 23) | mant
            F = orc.as_fp32(np.where(I >= 2 ** 31, I - 2 ** 32, I).astype(np.int32))
            n = np.arange(-E + 1, 255 - E, dtype=np.int64)          # -E < n < 255 - E
            got = orc.exponent_add(F[:, None], n[None, :])
            want = np.ldexp(F[:, None].astype(np.float64), n[None, :]).astype(np.float32)
            assert np.array_equal(got.view(np.int32), want.view(np.int32))


def test_lemma_random_normal_floats():
    rng = np.random.default_rng(2)
    I = rng.integers(-2 ** 31, 2 ** 31, 200000, dtype=np.int64).astype(np.int32)
    E = (I.astype(np.int64) >> 23) & 0xFF
    keep = (E > 0) & (E < 255)
    I, E = I[keep], E[keep]
    n = np.array([rng.integers(-e + 1, 255 - e) for e in E])
    F = orc.as_fp32(I)
    got = orc.exponent_add(F, n)
    want = (F.astype(np.float64) * np.exp2(n.astype(np.float64))).astype(np.float32)
    assert np.array_equal(got.view(np.int32), want.view(np.int32))


def test_unguarded_add_wraps_outside_the_range():
    """Why a guard is needed: 0.0 with n = -1 becomes a huge negative number."""
    bad = float(orc.exponent_add(np.float32(0.0), -1))
    assert bad < -1e30


def test_guarded_add_range_behaviour():
    rng = np.random.default_rng(3)
    I = rng.integers(-2 ** 31, 2 ** 31, 100000, dtype=np.int64).astype(np.int32)
    E = (I.astype(np.int64) >> 23) & 0xFF
    I = I[E < 255]
    F = orc.as_fp32(I)
    specials = np.array([0.0, -0.0, 1e-45, -1e-45, 1.1754944e-38, -1.1754944e-38, 2.0 ** -100], np.float32)
    F = np.concatenate([F, specials])
    for d in (0, -1, -2, -7, -30):
        got = orc.exponent_add_guarded(F, d)
        exact = F.astype(np.float64) * 2.0 ** d
        normal = np.abs(exact) >= 2.0 ** -126
        src_normal = np.abs(F.astype(np.float64)) >= 2.0 ** -126
        ok = normal & src_normal
        assert np.array_equal(got[ok].astype(np.float64), exact[ok])
        rest = ~ok
        assert np.all(np.abs(got[rest].astype(np.float64)) <= 2.0 ** -126)
        assert np.all(np.signbit(got) == np.signbit(F))


def test_exp_overflows_fp32_past_88():
    with np.errstate(over="ignore"):
        assert np.isfinite(np.exp(np.float32(88.0)))
        assert np.isinf(np.exp(np.float32(89.0)))


# ------------------------------------------------------------------ Algorithm 1 / Eq. (4)
def _problem(seed, G=6, L=333, sigma=1.0):
    rng = np.random.default_rng(seed)
    Q = rng.standard_normal((G, 576)) * sigma
    K = rng.standard_normal((L, 576))
    return Q, K, K[:, :512], 192 ** -0.5


def _chunks(L, size, rng=None):
    idx = [np.arange(lo, min(L, lo + size)) for lo in range(0, L, size)]
    if rng is not None:
        rng.shuffle(idx)
    return idx


@pytest.mark.parametrize("size", [1, 7, 64, 512, 333])
@pytest.mark.parametrize("shuffle", [False, True])
def test_algorithm1_chunk_size_and_order_invariance(size, shuffle):
    Q, K, V, scale = _problem(4)
    want, want_lse = orc.attention_rows(Q, K, scale)
    rng = np.random.default_rng(5) if shuffle else None
    O, m, l = orc.flash_attention(Q, K, V, scale, _chunks(len(K), size, rng))
    assert np.abs(O - want).max() < 1e-12
    assert np.abs(m + np.log(l) - want_lse).max() < 1e-12


@pytest.mark.parametrize("sigma", [1.0, 4.0, 10.0])
def test_amla_recurrence_equals_flash_attention(sigma):
    Q, K, V, scale = _problem(6, sigma=sigma)
    want, _ = orc.attention_rows(Q, K, scale)
    O, r = orc.amla_recurrence(Q, K, V, scale, _chunks(len(K), 64))
    assert np.abs(O - want).max() < 1e-12
    assert r.min() >= 2 ** -0.5 - 1e-12 and r.max() <= 2 ** 0.5 + 1e-12


def test_r_range_over_random_maxima():
    m = np.random.default_rng(7).uniform(-200, 200, 100000)
    n = np.rint(-m / math.log(2))
    r = np.exp(-n * math.log(2) - m)
    assert r.min() >= 2 ** -0.5 * (1 - 1e-12) and r.max() <= 2 ** 0.5 * (1 + 1e-12)


def test_fp32_emulation_with_exponent_add_tracks_definition():
    """Algorithm 2's loop in FP32 / BF16 P / INT32 add lands at the BF16-P error level."""
    rng = np.random.default_rng(8)
    def bf(x):
        return orc._round_bf16(x.astype(np.float32))
    for sigma in (1.0, 4.0):
        Q = bf(rng.standard_normal((16, 576)) * sigma)
        K = bf(rng.standard_normal((1000, 576)))
        want, want_lse = orc.attention_rows(Q.astype(np.float64), K.astype(np.float64), 192 ** -0.5)
        out, lse = orc.amla_fp32_emulation(Q, K, K[:, :512], 192 ** -0.5)
        assert np.abs(out - want).max() < 1e-2
        assert np.abs(lse - want_lse).max() < 1e-3
        assert orc.frobenius_error(out, want) < 4e-3


def test_lazy_reference_update_keeps_the_accuracy():
    """Deferring the reference until the max exceeds it by 2^8 changes nothing beyond rounding."""
    rng = np.random.default_rng(9)
    def bf(x):
        return orc._round_bf16(x.astype(np.float32))
    for sigma in (1.0, 4.0, 10.0):
        Q = bf(rng.standard_normal((16, 576)) * sigma)
        K = bf(rng.standard_normal((2000, 576)))
        want, want_lse = orc.attention_rows(Q.astype(np.float64), K.astype(np.float64), 192 ** -0.5)
        strict, _ = orc.amla_fp32_emulation(Q, K, K[:, :512], 192 ** -0.5)
        out, lse = orc.amla_fp32_emulation(Q, K, K[:, :512], 192 ** -0.5, lazy_threshold=8.0)
        assert np.abs(lse - want_lse).max() < 1e-3
        assert orc.frobenius_error(out, want) < 4e-3
        assert abs(orc.frobenius_error(out, want) - orc.frobenius_error(strict, want)) < 5e-4


def test_accuracy_level_matches_the_papers_table():
    """Section 5.1, Table 3, N(0,1) column: Base 1.77e-3 and AMLA 1.81e-3 relative Frobenius error
    against the high-precision result, outputs in BF16.  The paper does not state G, the scale or
    how V relates to K for that experiment, so this is a loose pin on the error *level* (the BF16
    rounding floor) and on "AMLA is nearly identical to Base": both emulations, with the output
    rounded to BF16, must land in 1.4e-3 .. 2.2e-3 and within 15 % of each other."""
    rng = np.random.default_rng(10)
    def bf(x):
        return orc._round_bf16(x.astype(np.float32))
    Q = bf(rng.standard_normal((32, 576)))
    K = bf(rng.standard_normal((8192, 576)))
    want, _ = orc.attention_rows(Q.astype(np.float64), K.astype(np.float64), 192 ** -0.5)
    base, _ = orc.flash_fp32_emulation(Q, K, K[:, :512], 192 ** -0.5)
    amla, _ = orc.amla_fp32_emulation(Q, K, K[:, :512], 192 ** -0.5)
    e_base = orc.frobenius_error(bf(base), want)
    e_amla = orc.frobenius_error(bf(amla), want)
    assert 1.4e-3 < e_base < 2.2e-3, e_base
    assert 1.4e-3 < e_amla < 2.2e-3, e_amla
    assert abs(e_amla - e_base) / e_base < 0.15


def _accuracy_sample(family, param, seed, rows=32, keys=8192):
    rng = np.random.default_rng(seed)
    draw = (lambda shape: rng.standard_normal(shape) * param) if family == "n" else \
           (lambda shape: rng.uniform(-param, param, shape))
    Q = orc._round_bf16(draw((rows, 576)).astype(np.float32))
    K = orc._round_bf16(draw((keys, 576)).astype(np.float32))
    return Q, K


@pytest.mark.parametrize("family,param,base_printed,amla_printed",
                         [(f, float(p), float(b), float(a)) for f, p, b, a in _rows("table3_table4_accuracy.txt")])
def test_emulations_reproduce_the_printed_accuracy_tables(family, param, base_printed, amla_printed):
    """Tables 3 and 4: the FP32 emulation of Algorithm 1 ("Base") and the step-by-step emulation of
    Algorithm 2 with Appendix A's c_i ("AMLA"), outputs rounded to BF16, land on the printed errors:
    within 1.5 % on the two flat columns N(0,1) and U(-1,1), where one sample of 32 rows already has
    0.5 % spread and the printed AMLA-minus-Base gap of 2 % is resolved, and within 7 % (mean of three
    samples; the spread of one sample is 2-6 %) on the others.  With Algorithm 2's c_i as printed the same
    emulation gives 3.1e-3 on N(0,1), 70 % above the printed 1.81e-3."""
    scale = 576 ** -0.5
    flat = param == 1.0
    e_base, e_amla = [], []
    for seed in ((100,) if flat else (100, 101, 102)):
        Q, K = _accuracy_sample(family, param, seed)
        V = K[:, :512]
        want, _ = orc.attention_rows(Q.astype(np.float64), K.astype(np.float64), scale)
        e = lambda x: orc.frobenius_error(orc._round_bf16(np.asarray(x, dtype=np.float32)), want)
        e_base.append(e(orc.flash_fp32_emulation(Q, K, V, scale, block=512)[0]))
        e_amla.append(e(orc.amla_alg2_emulation(Q, K, V, scale, block=512)))
        if flat and family == "n":
            printed_c = e(orc.amla_alg2_emulation(Q, K, V, scale, block=512, c_reading="algorithm"))
            assert printed_c > 1.5 * amla_printed, printed_c
    tol = 0.015 if flat else 0.07
    assert abs(np.mean(e_base) - base_printed) < tol * base_printed, (np.mean(e_base), base_printed)
    assert abs(np.mean(e_amla) - amla_printed) < tol * amla_printed, (np.mean(e_amla), amla_printed)
    if flat:
        assert e_amla[0] > e_base[0]          # the printed ordering on these columns


def test_algorithm2_compensation_and_the_two_readings_of_c():
    """Algorithm 2 prints c_i = S32 / S16, Appendix A defines c_i = r_i / r'_i = S16 / S32.  With
    the appendix's definition the compensated recurrence, outputs rounded to BF16, is as accurate as
    Base (what Tables 3-4 report); with the printed one the correction has the wrong sign and the
    error before output rounding is more than twice as large.  Without any compensation (power-of-two
    reference, largest weight not BF16-exact) the error on peaked rows is 25-40 % above Base when one
    FP32 row sum normalises the output; the kernels' ADD and lazy variants keep a second sum over the
    rounded weights, which takes most of that back (3-12 % above Base on 32-row means; 25 % is this 16-row sample's bound).  Value rows are
    nonzero here (the raw INT32 add of Algorithm 2 has no guard for zeros)."""
    rng = np.random.default_rng(11)
    def bf(x):
        return orc._round_bf16(x.astype(np.float32))
    for sigma in (1.0, 2.0, 4.0):
        Q = bf(rng.standard_normal((16, 576)) * sigma)
        K = bf(rng.standard_normal((4096, 576)))
        want, _ = orc.attention_rows(Q.astype(np.float64), K.astype(np.float64), 192 ** -0.5)
        e = lambda x: orc.frobenius_error(x, want)
        app = orc.amla_alg2_emulation(Q, K, K[:, :512], 192 ** -0.5, c_reading="appendix")
        alg = orc.amla_alg2_emulation(Q, K, K[:, :512], 192 ** -0.5, c_reading="algorithm")
        base, _ = orc.flash_fp32_emulation(Q, K, K[:, :512], 192 ** -0.5)
        one_sum, _ = orc.amla_fp32_emulation(Q, K, K[:, :512], 192 ** -0.5)
        two_sums, _ = orc.amla_fp32_emulation(Q, K, K[:, :512], 192 ** -0.5, normalise="b16")
        lazy, _ = orc.amla_fp32_emulation(Q, K, K[:, :512], 192 ** -0.5, normalise="b16", lazy_threshold=8)
        assert e(alg) > 1.9 * e(app), (sigma, e(alg), e(app))
        assert abs(e(bf(app)) - e(bf(base))) < 0.1 * e(bf(base)), (sigma, e(bf(app)), e(bf(base)))
        assert e(bf(base)) <= e(bf(one_sum)) < 1.8 * e(bf(base)), (sigma, e(bf(one_sum)), e(bf(base)))
        assert e(bf(two_sums)) < 1.25 * e(bf(base)), (sigma, e(bf(two_sums)), e(bf(base)))
        assert e(bf(lazy)) < 1.25 * e(bf(base)), (sigma, e(bf(lazy)), e(bf(base)))
        if sigma > 1.0:
            assert e(bf(two_sums)) < 0.95 * e(bf(one_sum)), (sigma, e(bf(two_sums)), e(bf(one_sum)))


def test_compensation_restated_in_base_two_matches_algorithm2():
    """The one-reference-per-row form (ref = m - log2 S16, N built in integers, two row sums) is the
    same method as Algorithm 2 step by step: its error against the fp64 definition is the step-by-step
    emulation's and Base's within a few per cent, its lse is the definition's, and dropping the
    mantissa term eps makes flat rows (many small maxima updates, no dominant key) measurably worse."""
    rng = np.random.default_rng(12)
    def bf(x):
        return orc._round_bf16(x.astype(np.float32))
    for sigma in (1.0, 4.0):
        Q = bf(rng.standard_normal((16, 576)) * sigma)
        K = bf(rng.standard_normal((4096, 576)))
        V = K[:, :512]
        want, want_lse = orc.attention_rows(Q.astype(np.float64), K.astype(np.float64), 192 ** -0.5)
        e = lambda x: orc.frobenius_error(bf(x), want)
        comp, lse = orc.amla_comp_fp32_emulation(Q, K, V, 192 ** -0.5)
        alg2 = orc.amla_alg2_emulation(Q, K, V, 192 ** -0.5, block=64)
        base, _ = orc.flash_fp32_emulation(Q, K, V, 192 ** -0.5)
        assert abs(e(comp) - e(alg2)) < 0.03 * e(alg2), (sigma, e(comp), e(alg2))
        assert abs(e(comp) - e(base)) < 0.06 * e(base), (sigma, e(comp), e(base))
        assert np.abs(lse - want_lse).max() < 2e-5
        assert np.abs(comp.astype(np.float64) - want).max() < 1e-2
        if sigma == 1.0:
            no_eps, _ = orc.amla_comp_fp32_emulation(Q, K, V, 192 ** -0.5, with_eps=False)
            assert e(no_eps) > 1.05 * e(comp), (e(no_eps), e(comp))


def test_compensation_survives_zero_values_and_the_clamp():
    """Zero value columns stay at most a few subnormal steps from zero under the guarded add (a
    positive mantissa term turns the bit pattern 0 into a subnormal, a negative one is caught by the
    guard), and a row max that jumps by far more than 2^30 between blocks (old accumulator
    irrelevant) still gives the definition's result."""
    rng = np.random.default_rng(13)
    def bf(x):
        return orc._round_bf16(x.astype(np.float32))
    Q = bf(rng.standard_normal((8, 576)) * 3)
    K = bf(rng.standard_normal((512, 576)))
    K[300] = bf(Q[0] * 4)             # a late key far above everything before it for row 0
    K[:, 5] = 0.0
    want, want_lse = orc.attention_rows(Q.astype(np.float64), K.astype(np.float64), 192 ** -0.5)
    out, lse = orc.amla_comp_fp32_emulation(Q, K, K[:, :512], 192 ** -0.5)
    assert np.all(np.abs(out[:, 5]) < 2.0 ** -126)
    assert np.abs(out.astype(np.float64) - want).max() < 1e-2 * max(1.0, np.abs(want).max())
    assert np.abs(lse - want_lse).max() < 1e-4


# -------------------------------------------------------------------- accounting pins
def test_table2_arithmetic_intensity():
    for name, qh, kvh, sq, printed, kind in _rows("table2_arithmetic_intensity.txt"):
        qh, kvh, sq, printed = int(qh), int(kvh), int(sq), float(printed)
        S2 = 4096
        if kind == "mla":
            ai = acc.decode_flops(qh, sq, S2) / acc.kv_bytes_mla(S2)
        else:
            ai = acc.decode_flops(qh, sq, S2, 128, 128) / acc.kv_bytes_mha_gqa(kvh, S2, 128, 128)
        assert abs(ai - printed) <= 0.5 + 0.005 * printed, (name, ai)


def test_table5_durations_reproduce_printed_utilisation():
    rows = [(int(a), int(b), float(c), float(d)) for a, b, c, d in _rows("table5_ascend_rows.txt")]
    batch, heads = 96, 128
    best = [r for r in rows if r[0] == 2 and r[1] == 16384][0]
    tflops_best = acc.decode_flops(heads, 2, batch * 16384) / (best[2] * 1e-6) / 1e12
    assert abs(tflops_best - 614) < 1.0                       # the abstract's 614 TFLOPS
    peak = tflops_best / (best[3] / 100)
    for sq, sk, dur, fu in rows:
        tf = acc.decode_flops(heads, sq, batch * sk) / (dur * 1e-6) / 1e12
        assert abs(tf / peak * 100 - fu) < 0.6, (sq, sk, tf / peak * 100, fu)


def test_frobenius_error_metric():
    A = np.array([[3.0, 0.0], [0.0, 4.0]])
    B = np.zeros((2, 2))
    assert orc.frobenius_error(B, A) == pytest.approx(1.0, abs=1e-9)
    assert orc.frobenius_error(A, A) == 0.0


def test_guarded_add_boundary_cases():
    # E + n < 0 -> signed zero; E + n == 0 -> mantissa bits only; E + n > 0 -> exact product
    one_and_half_min = np.float32(1.5 * 2.0 ** -126)            # E = 1, M = 2^22
    got = orc.exponent_add_guarded(np.array([one_and_half_min, -one_and_half_min], np.float32), -1)
    assert got.view(np.uint32).tolist() == [0x00400000, 0x80400000]
    got = orc.exponent_add_guarded(np.array([one_and_half_min, -one_and_half_min, 0.0, -0.0], np.float32), -2)
    assert got.view(np.uint32).tolist() == [0x00000000, 0x80000000, 0x00000000, 0x80000000]
    got = orc.exponent_add_guarded(np.array([3.0, -3.0], np.float32), -30)
    assert got.tolist() == [3.0 * 2.0 ** -30, -3.0 * 2.0 ** -30]
