"""amla_decode_static_workspace, the entry point for callers that cannot allocate device memory, against
amla_decode on the same inputs: same kernels, so the outputs are compared bit for bit (which is inside the
parity bar amla_decode itself is held to against the oracle).  Two calls in a row share the library's static
array, the second with a smaller input whose partial results cover only the array's beginning: stale contents
of the first call must not reach the second call's output.  Oversized requests are refused."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2509_25224_amd import amla, workloads as wl
    return torch, amla, wl


def _dev(torch, case):
    dev = torch.device("cuda:0")
    q = torch.from_numpy(case.q_bits.view(np.int16)).to(dev).view(torch.bfloat16)
    kv = torch.from_numpy(case.kv_bits.view(np.int16)).to(dev).view(torch.bfloat16)
    return q, kv, torch.from_numpy(case.block_table).to(dev), torch.from_numpy(case.seqlens).to(dev)


def _pair(torch, amla, case, variant, flags, ns):
    q, kv, tab, lens = _dev(torch, case)
    want, want_lse = amla.amla_decode(q, kv, tab, lens, case.softmax_scale, variant=variant, flags=flags, num_splits=ns)
    out = torch.full_like(want, float("nan"))
    lse = torch.full_like(want_lse, float("nan"))
    before = torch.cuda.memory_allocated()
    amla.amla_decode_static_workspace(q, kv, tab, lens, case.softmax_scale, out, lse, variant=variant, flags=flags,
                                      num_splits=ns)
    assert torch.cuda.memory_allocated() == before          # torch's allocator was not asked for anything either
    torch.cuda.synchronize()
    return out, lse, want, want_lse


@pytest.mark.parametrize("variant,flags,ns", [(1, 0, 4), (0, 8, 24), (2, 0, 3), (1, 128, 4)],
                         ids=["add_splits", "mul_balanced", "add_comp_splits", "add_transposed_splits"])
def test_two_calls_in_a_row_the_second_smaller(env, variant, flags, ns):
    torch, amla, wl = env
    first = wl.make_case("first", 71, batch=6, s_q=2, heads=128, seqlens=[900, 64, 1, 2000, 0, 513], spare_frac=0.25)
    second = wl.make_case("second", 72, batch=2, s_q=1, heads=128, seqlens=[700, 130])
    for case in (first, second):
        d = amla.make_desc(case.batch, case.s_q, case.heads, case.num_blocks, case.max_blocks_per_seq, variant, ns, flags)
        assert 0 < amla.amla_workspace_bytes(d) <= amla.amla_static_workspace_limit()
        out, lse, want, want_lse = _pair(torch, amla, case, variant, flags, ns)
        assert torch.equal(out.view(torch.int16), want.view(torch.int16)), case.name
        assert torch.equal(lse.view(torch.int32), want_lse.view(torch.int32)), case.name


def test_shape_that_needs_no_workspace(env):
    torch, amla, wl = env
    case = wl.make_config(0)
    out, lse, want, want_lse = _pair(torch, amla, case, 1, 0, 1)
    assert torch.equal(out.view(torch.int16), want.view(torch.int16))
    assert torch.equal(lse.view(torch.int32), want_lse.view(torch.int32))


def test_largest_measured_workspace_fits_and_matches(env):
    """The balanced decomposition of the 128-sequence, two-token batch asks for 127.7 MiB, the most of all
    measured configurations: it fits the 128 MiB array."""
    torch, amla, wl = env
    case = wl.make_config(2)
    d = amla.make_desc(case.batch, case.s_q, case.heads, case.num_blocks, case.max_blocks_per_seq, 1, 0, amla.AMLA_FLAG_BALANCED)
    assert amla.amla_workspace_bytes(d) <= amla.amla_static_workspace_limit() == 128 << 20
    out, lse, want, want_lse = _pair(torch, amla, case, 1, amla.AMLA_FLAG_BALANCED, 0)
    assert torch.equal(out.view(torch.int16), want.view(torch.int16))
    assert torch.equal(lse.view(torch.int32), want_lse.view(torch.int32))


def test_request_beyond_the_array_is_refused(env):
    torch, amla, wl = env
    case = wl.make_case("big", 73, batch=20, s_q=2, heads=128, seqlens=[64] * 20)
    q, kv, tab, lens = _dev(torch, case)
    out = torch.zeros((case.batch, case.s_q, case.heads, 512), dtype=torch.bfloat16, device="cuda:0")
    d = amla.make_desc(case.batch, case.s_q, case.heads, case.num_blocks, case.max_blocks_per_seq, 1, 16, 0)
    assert amla.amla_workspace_bytes(d) > amla.amla_static_workspace_limit()
    with pytest.raises(amla.AmlaError) as e:
        amla.amla_decode_static_workspace(q, kv, tab, lens, case.softmax_scale, out, None, variant=1, num_splits=16)
    assert e.value.status == amla.AMLA_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((out == 0).all())                             # nothing was enqueued
