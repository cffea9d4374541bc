"""GPU parity of the eight-wave equal-share kernel (AMLA_FLAG_EIGHT_WAVES: 16 rows per wave, two waves per
SIMD, v_mfma_f32_16x16x32_bf16).  Its operand layouts are the documented ones and have not been measured by
this build yet, so the first case is the smallest one; a wrong layout shows as a wrong result there, not as a
fault (every address the kernel forms is the same set the default kernel reads).  Collected after the files
whose cases have run on the GPU."""
import numpy as np
import pytest

from test_gpu_parity import ADD, LAZY, LSE_TOL, MUL, check, env, out_tolerance, run_gpu, to_dev  # noqa: F401

pytestmark = pytest.mark.gpu

COMP = 2
LDEXP = 3
W8 = 64
KINDS = [pytest.param((MUL, 0), id="mul"), pytest.param((ADD, 0), id="add"), pytest.param((MUL, LAZY), id="mul_lazy"),
         pytest.param((ADD, LAZY), id="add_lazy"), pytest.param((LDEXP, 0), id="add_ldexp"),
         pytest.param((LDEXP, LAZY), id="add_ldexp_lazy"), pytest.param((COMP, 0), id="add_comp")]


@pytest.mark.parametrize("kind", KINDS)
def test_tiny_config_eight_waves(env, kind):
    torch, orc, amla, wl = env
    case = wl.make_config(0)
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    out, lse = run_gpu(torch, amla, case, to_dev(torch, case), variant=kind[0], flags=kind[1] | W8)
    check(out, lse, want, want_lse, f"tiny eight waves {kind}")


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("splits", [1, 3])
def test_ragged_eight_waves(env, kind, splits):
    """Partial last blocks, a one-key sequence, rows past the end of the row range (80 heads x 2 tokens in
    128-row tiles), split and unsplit."""
    torch, orc, amla, wl = env
    case = wl.make_case("edges", 21, batch=6, s_q=2, heads=80, seqlens=[1, 63, 64, 65, 300, 1000], spare_frac=0.25)
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    out, lse = run_gpu(torch, amla, case, to_dev(torch, case), variant=kind[0], flags=kind[1] | W8, num_splits=splits)
    check(out, lse, want, want_lse, f"edges eight waves splits={splits} {kind}")


@pytest.mark.parametrize("kind", [pytest.param((MUL, LAZY), id="mul_lazy"), pytest.param((ADD, LAZY), id="add_lazy")])
def test_wide_logits_eight_waves(env, kind):
    torch, orc, amla, wl = env
    case = wl.make_case("wide", 22, batch=2, s_q=2, heads=64, seqlens=[3000, 4500], q_sigma=4.0)
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    out, lse = run_gpu(torch, amla, case, to_dev(torch, case), variant=kind[0], flags=kind[1] | W8)
    half_ulp = 2.0 ** (np.ceil(np.log2(np.maximum(np.abs(want), 2.0 ** -20))) - 9)
    assert np.all(np.abs(out - want) <= half_ulp + 6e-3)
    assert np.abs(lse - want_lse).max() <= LSE_TOL


@pytest.mark.parametrize("kind", [pytest.param((ADD, 0), id="add"), pytest.param((MUL, 0), id="mul")])
def test_headline_shape_eight_waves(env, kind):
    """The benchmark's configuration (batch 128, s_q 2, 128 heads, kv 4096), all rows against the oracle
    sequence by sequence."""
    torch, orc, amla, wl = env
    case = wl.make_config(2)
    out, lse = run_gpu(torch, amla, case, to_dev(torch, case), variant=kind[0], flags=kind[1] | W8)
    worst = [0.0, 0.0]
    for b in range(case.batch):
        want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens,
                                    case.softmax_scale, seq_ids=[b])
        assert np.all(np.abs(out[b] - want[b]) <= out_tolerance(want[b])), (b, kind)
        worst[0] = max(worst[0], float(np.abs(out[b] - want[b]).max()))
        worst[1] = max(worst[1], float(np.abs(lse[b] - want_lse[b]).max()))
    print(f"config 2 eight waves {kind}: max|out err| {worst[0]:.3e} max|lse err| {worst[1]:.3e}", flush=True)
    assert worst[1] <= LSE_TOL


@pytest.mark.parametrize("family,param,base_printed,amla_printed", [("n", 1.0, 1.77e-3, 1.81e-3), ("u", 1.0, 1.97e-3, 2.01e-3)])
def test_accuracy_tables_eight_waves(env, family, param, base_printed, amla_printed):
    """Section 5.1's experiment (Tables 3 and 4, the two flat columns) through the eight-wave MUL ('Base')
    and compensated ('AMLA') kernels."""
    torch, orc, amla, wl = env
    case = wl.make_accuracy_case(family, param)
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    dev = to_dev(torch, case)
    for variant, printed in ((MUL, base_printed), (COMP, amla_printed)):
        out, lse = run_gpu(torch, amla, case, dev, variant=variant, flags=W8, num_splits=1)
        err = orc.frobenius_error(out.reshape(-1, 512), want.reshape(-1, 512))
        print(f"{family} {param:g} eight waves v{variant}: {err:.3e} (printed {printed:.2e})", flush=True)
        assert abs(err - printed) < 0.03 * printed, (variant, err)
        assert np.abs(lse - want_lse).max() <= LSE_TOL
