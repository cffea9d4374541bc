"""GPU parity of the ADD_COMP variant (Algorithm 2 with its BF16 scale compensation, the steps from S32 to N,
and Appendix A) in both kernel families, and of the ldexp form of the exponent add."""
import numpy as np
import pytest

from test_gpu_parity import (ADD, COMP, LSE_TOL, MUL, TRANSPOSED, check, env, out_tolerance, run_gpu, to_dev)  # noqa: F401

pytestmark = pytest.mark.gpu

FAMILY = [pytest.param(0, id="row"), pytest.param(TRANSPOSED, id="transposed")]


@pytest.mark.parametrize("family", FAMILY)
def test_tiny_config_comp(env, family):
    torch, orc, amla, wl = env
    assert amla.AMLA_RESCALE_ADD_COMP == COMP
    case = wl.make_config(0)
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    out, lse = run_gpu(torch, amla, case, to_dev(torch, case), variant=COMP, flags=family)
    check(out, lse, want, want_lse, "tiny comp")


@pytest.mark.parametrize("family", FAMILY)
@pytest.mark.parametrize("splits", [1, 3])
def test_ragged_comp(env, splits, family):
    torch, orc, amla, wl = env
    case = wl.make_case("edges", 31, batch=6, s_q=2, heads=80, seqlens=[1, 63, 64, 65, 300, 1000], spare_frac=0.25)
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    out, lse = run_gpu(torch, amla, case, to_dev(torch, case), variant=COMP, num_splits=splits, flags=family)
    check(out, lse, want, want_lse, f"edges comp splits={splits}")


@pytest.mark.parametrize("family", FAMILY)
@pytest.mark.parametrize("sigma", [4.0, 10.0])
def test_wide_logits_comp(env, sigma, family):
    """Peaked rows with many row-max updates: every update changes c_i, so the mantissa term of the
    integer add is exercised with both signs, and jumps of more than 30 binades hit the clamp."""
    torch, orc, amla, wl = env
    case = wl.make_case("wide", 32, batch=2, s_q=2, heads=64, seqlens=[3000, 4500], q_sigma=sigma)
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    out, lse = run_gpu(torch, amla, case, to_dev(torch, case), variant=COMP, flags=family)
    assert np.all(np.abs(out - want) <= out_tolerance(want))       # the compensated weights: the flat bound holds
    assert np.abs(lse - want_lse).max() <= LSE_TOL


@pytest.mark.parametrize("family", FAMILY)
def test_comp_is_as_accurate_as_mul(env, family):
    """What the compensation is for (Section 3.2, Tables 3-4): the relative Frobenius error of ADD_COMP
    against the fp64 definition equals that of the MUL variant (Algorithm 1's arithmetic) within a
    few per cent, on flat rows and on peaked rows, where the plain ADD variant is measurably worse."""
    torch, orc, amla, wl = env
    for sigma in (1.0, 4.0):
        case = wl.make_case("acc", 33, batch=2, s_q=1, heads=128, seqlens=[8192, 8192], q_sigma=sigma)
        want, _ = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
        dev = to_dev(torch, case)
        err = {}
        for name, v in (("mul", MUL), ("add", ADD), ("comp", COMP)):
            out, _ = run_gpu(torch, amla, case, dev, variant=v, flags=family)
            err[name] = orc.frobenius_error(out.reshape(-1, 512), want.reshape(-1, 512))
        print(f"sigma {sigma}: E mul {err['mul']:.3e} add {err['add']:.3e} comp {err['comp']:.3e}", flush=True)
        assert abs(err["comp"] - err["mul"]) < 0.10 * err["mul"], err
        assert err["comp"] <= err["add"] * 1.05, err


@pytest.mark.parametrize("family", FAMILY)
def test_zero_value_columns_stay_negligible_comp(env, family):
    torch, orc, amla, wl = env
    case = wl.make_case("zeros", 34, batch=2, s_q=1, heads=64, seqlens=[700, 1500], q_sigma=3.0)
    case.kv_bits[:, :, 7] = 0
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    out, lse = run_gpu(torch, amla, case, to_dev(torch, case), variant=COMP, flags=family)
    assert np.all(np.abs(out[..., 7]) < 2.0 ** -100)
    check(out, lse, want, want_lse, "zeros comp")


# ---- the ADD variant with the exponent add done by v_ldexp_f32 (AMLA_RESCALE_ADD_LDEXP) ----------------
LDEXP = 3
LAZY_FLAG = 2


@pytest.mark.parametrize("flags", [0, LAZY_FLAG])
@pytest.mark.parametrize("splits", [1, 3])
def test_ldexp_variant_small_cases(env, flags, splits):
    torch, orc, amla, wl = env
    assert amla.AMLA_RESCALE_ADD_LDEXP == LDEXP
    case = wl.make_case("edges", 35, batch=6, s_q=2, heads=80, seqlens=[1, 63, 64, 65, 300, 1000], spare_frac=0.25)
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    out, lse = run_gpu(torch, amla, case, to_dev(torch, case), variant=LDEXP, flags=flags, num_splits=splits)
    check(out, lse, want, want_lse, f"edges ldexp flags={flags} splits={splits}")


def test_ldexp_variant_headline_shape(env):
    torch, orc, amla, wl = env
    case = wl.make_config(2)
    out, lse = run_gpu(torch, amla, case, to_dev(torch, case), variant=LDEXP)
    worst = [0.0, 0.0]
    for b in range(0, case.batch, 8):
        want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens,
                                    case.softmax_scale, seq_ids=[b])
        assert np.all(np.abs(out[b] - want[b]) <= out_tolerance(want[b])), b
        worst[0] = max(worst[0], float(np.abs(out[b] - want[b]).max()))
        worst[1] = max(worst[1], float(np.abs(lse[b] - want_lse[b]).max()))
    print(f"config 2 ldexp: max|out err| {worst[0]:.3e} max|lse err| {worst[1]:.3e}", flush=True)
    assert worst[1] <= LSE_TOL


def test_ldexp_variant_equals_the_integer_add(env):
    """Inside Lemma 3.1's range the two forms of the exponent add are the same operation: same reference,
    same weights, same products, so the strict ADD and ADD_LDEXP outputs agree bit for bit on inputs whose
    accumulators stay normal (N(0,1) data; kv 4096)."""
    torch, orc, amla, wl = env
    case = wl.make_case("same", 36, batch=2, s_q=1, heads=128, seqlens=[4096, 4096])
    dev = to_dev(torch, case)
    a, la = run_gpu(torch, amla, case, dev, variant=ADD, flags=TRANSPOSED)
    b, lb = run_gpu(torch, amla, case, dev, variant=LDEXP)
    assert np.array_equal(a, b) and np.array_equal(la, lb)
