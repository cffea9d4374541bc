"""GPU parity of the lazy reference update (AMLA_FLAG_LAZY_RESCALE; transposed-accumulator kernels): the
reference of the exponent moves only when the row max exceeds it by more than 2^8."""
import numpy as np
import pytest

from test_gpu_parity import (ADD, LAZY, LSE_TOL, MUL, check, env, out_tolerance, run_gpu, to_dev)  # noqa: F401

pytestmark = pytest.mark.gpu

BOTH = [pytest.param(MUL, id="mul_lazy"), pytest.param(ADD, id="add_lazy")]


@pytest.mark.parametrize("variant", BOTH)
def test_tiny_config_lazy(env, variant):
    torch, orc, amla, wl = env
    case = wl.make_config(0)
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    out, lse = run_gpu(torch, amla, case, to_dev(torch, case), variant=variant, flags=LAZY)
    check(out, lse, want, want_lse, f"tiny lazy v{variant}")


@pytest.mark.parametrize("variant", BOTH)
@pytest.mark.parametrize("splits", [1, 3])
def test_ragged_lazy(env, variant, splits):
    torch, orc, amla, wl = env
    case = wl.make_case("edges", 21, batch=6, s_q=2, heads=80, seqlens=[1, 63, 64, 65, 300, 1000], spare_frac=0.25)
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    out, lse = run_gpu(torch, amla, case, to_dev(torch, case), variant=variant, flags=LAZY, num_splits=splits)
    check(out, lse, want, want_lse, f"edges lazy splits={splits} v{variant}")


@pytest.mark.parametrize("variant", BOTH)
@pytest.mark.parametrize("sigma", [4.0, 10.0])
def test_wide_logits_cross_the_threshold(env, variant, sigma):
    """Logit spread of tens of base-2 units: the row max outruns the reference by more than 2^8
    several times, so both the deferred and the taken update are exercised."""
    torch, orc, amla, wl = env
    case = wl.make_case("wide", 22, batch=2, s_q=2, heads=64, seqlens=[3000, 4500], q_sigma=sigma)
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    out, lse = run_gpu(torch, amla, case, to_dev(torch, case), variant=variant, flags=LAZY)
    half_ulp = 2.0 ** (np.ceil(np.log2(np.maximum(np.abs(want), 2.0 ** -20))) - 9)
    assert np.all(np.abs(out - want) <= half_ulp + 6e-3)
    assert np.abs(lse - want_lse).max() <= LSE_TOL


@pytest.mark.parametrize("index", [2])
def test_full_size_lazy(env, index):
    torch, orc, amla, wl = env
    case = wl.make_config(index)
    dev = to_dev(torch, case)
    res = {v: run_gpu(torch, amla, case, dev, variant=v, flags=LAZY) for v in (MUL, ADD)}
    worst = {v: [0.0, 0.0] for v in res}
    for b in range(case.batch):
        want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens,
                                    case.softmax_scale, seq_ids=[b])
        for v, (out, lse) in res.items():
            assert np.all(np.abs(out[b] - want[b]) <= out_tolerance(want[b])), (index, b, v)
            worst[v][0] = max(worst[v][0], float(np.abs(out[b] - want[b]).max()))
            worst[v][1] = max(worst[v][1], float(np.abs(lse[b] - want_lse[b]).max()))
    for v in res:
        print(f"config {index} lazy variant {v}: max|out err| {worst[v][0]:.3e} max|lse err| {worst[v][1]:.3e}",
              flush=True)
        assert worst[v][1] <= LSE_TOL
