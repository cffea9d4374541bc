"""GPU parity of the prefetching build of the compiler kernels' loop (AMLA_FLAG_PREFETCH: the LDS operand
reads of both products issued ahead of their use).  The arithmetic and its order are those of the
plain kernels, so each case is checked twice: against the oracle with the usual bounds, and bit for bit
against the plain kernel of the same variant.  Collected after the files whose cases have run on the GPU."""
import numpy as np
import pytest

from test_gpu_parity import ADD, LAZY, LSE_TOL, MUL, check, env, out_tolerance, run_gpu, to_dev  # noqa: F401

pytestmark = pytest.mark.gpu

LDEXP = 3
PREFETCH = 32
KINDS = [pytest.param((MUL, 0), id="mul"), pytest.param((ADD, 0), id="add"), pytest.param((MUL, LAZY), id="mul_lazy"),
         pytest.param((ADD, LAZY), id="add_lazy"), pytest.param((LDEXP, 0), id="add_ldexp"),
         pytest.param((LDEXP, LAZY), id="add_ldexp_lazy")]


def both(torch, amla, case, kind, **kw):
    dev = to_dev(torch, case)
    plain = run_gpu(torch, amla, case, dev, variant=kind[0], flags=kind[1], **kw)
    ahead = run_gpu(torch, amla, case, dev, variant=kind[0], flags=kind[1] | PREFETCH, **kw)
    return plain, ahead


@pytest.mark.parametrize("kind", KINDS)
def test_tiny_config_prefetch(env, kind):
    torch, orc, amla, wl = env
    case = wl.make_config(0)
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    plain, ahead = both(torch, amla, case, kind)
    check(ahead[0], ahead[1], want, want_lse, f"tiny prefetch {kind}")
    assert np.array_equal(plain[0], ahead[0]) and np.array_equal(plain[1], ahead[1])


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("splits", [1, 3])
def test_ragged_prefetch(env, kind, splits):
    """Partial last blocks, a one-key sequence, rows past the end of the row range (80 heads x 2 tokens in
    128-row tiles), split and unsplit."""
    torch, orc, amla, wl = env
    case = wl.make_case("edges", 21, batch=6, s_q=2, heads=80, seqlens=[1, 63, 64, 65, 300, 1000], spare_frac=0.25)
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    plain, ahead = both(torch, amla, case, kind, num_splits=splits)
    check(ahead[0], ahead[1], want, want_lse, f"edges prefetch splits={splits} {kind}")
    assert np.array_equal(plain[0], ahead[0]) and np.array_equal(plain[1], ahead[1])


@pytest.mark.parametrize("kind", [pytest.param((ADD, 0), id="add"), pytest.param((MUL, 0), id="mul")])
def test_headline_shape_prefetch(env, kind):
    """The benchmark's configuration (batch 128, s_q 2, 128 heads, kv 4096), all rows against the oracle
    sequence by sequence, and bit for bit against the plain kernel."""
    torch, orc, amla, wl = env
    case = wl.make_config(2)
    plain, ahead = both(torch, amla, case, kind)
    out, lse = ahead
    worst = [0.0, 0.0]
    for b in range(case.batch):
        want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens,
                                    case.softmax_scale, seq_ids=[b])
        assert np.all(np.abs(out[b] - want[b]) <= out_tolerance(want[b])), (b, kind)
        worst[0] = max(worst[0], float(np.abs(out[b] - want[b]).max()))
        worst[1] = max(worst[1], float(np.abs(lse[b] - want_lse[b]).max()))
    print(f"config 2 prefetch {kind}: max|out err| {worst[0]:.3e} max|lse err| {worst[1]:.3e}", flush=True)
    assert worst[1] <= LSE_TOL
    assert np.array_equal(plain[0], ahead[0]) and np.array_equal(plain[1], ahead[1])
