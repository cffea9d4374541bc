"""GPU parity of the balanced decomposition (AMLA_FLAG_BALANCED): the batch's blocks laid end to end
and cut into equal worker ranges, pieces merged per sequence; the causal mask among the s_q tokens and
per-sequence query counts, which live in the same kernels.  Both kernel families.  The integer arithmetic
itself is covered on the CPU by tests/test_plan.py."""
import numpy as np
import pytest

from test_gpu_parity import ADD, COMP, LAZY, LSE_TOL, MUL, TRANSPOSED, check, env, out_tolerance, run_gpu, to_dev  # noqa: F401

pytestmark = pytest.mark.gpu

BALANCED = 8
CAUSAL = 16
KINDS = [pytest.param((MUL, 0), id="mul"), pytest.param((ADD, 0), id="add"), pytest.param((COMP, 0), id="add_comp"),
         pytest.param((MUL, TRANSPOSED), id="mul_t"), pytest.param((ADD, TRANSPOSED), id="add_t"),
         pytest.param((ADD, LAZY), id="add_lazy"), pytest.param((COMP, TRANSPOSED), id="add_comp_t")]


@pytest.mark.parametrize("kind", KINDS)
def test_tiny_config_balanced(env, kind):
    torch, orc, amla, wl = env
    case = wl.make_config(0)
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    out, lse = run_gpu(torch, amla, case, to_dev(torch, case), variant=kind[0], flags=kind[1] | BALANCED)
    check(out, lse, want, want_lse, f"tiny balanced {kind}")


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("workers", [0, 1, 3, 8, 41])
def test_ragged_balanced(env, kind, workers):
    """Lengths 0, 1, 63, 64, 65 and a few hundred to a thousand keys, 160 rows (two row tiles, the second
    ragged), worker counts below, at and above the number of sequences, and one (41) above the
    number of blocks."""
    torch, orc, amla, wl = env
    case = wl.make_case("edges", 41, batch=7, s_q=2, heads=80, seqlens=[1, 63, 0, 64, 65, 300, 1000], spare_frac=0.25)
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    out, lse = run_gpu(torch, amla, case, to_dev(torch, case), variant=kind[0], flags=kind[1] | BALANCED,
                       num_splits=workers)
    check(out, lse, want, want_lse, f"edges balanced workers={workers} {kind}")


def test_balanced_matches_equal_share_split_on_a_uniform_batch(env):
    """On equal lengths with workers = sequences * splits the two decompositions cut at the same
    blocks and merge in the same order; the outputs then agree to within one bf16 step and the lse to
    FP32 rounding."""
    torch, orc, amla, wl = env
    case = wl.make_case("uniform", 42, batch=4, s_q=1, heads=128, seqlens=[2048] * 4)
    dev = to_dev(torch, case)
    a, la = run_gpu(torch, amla, case, dev, variant=ADD, num_splits=4)
    b, lb = run_gpu(torch, amla, case, dev, variant=ADD, num_splits=16, flags=BALANCED)
    assert np.all(np.abs(a - b) <= 2.0 ** -8 * np.maximum(np.abs(a), 2.0 ** -6))
    assert np.abs(la - lb).max() <= 1e-6


def test_full_size_ragged_config_balanced(env):
    """The ragged configuration (batch 32, kv_len 1024 .. 16384) under the balanced decomposition, every row."""
    torch, orc, amla, wl = env
    case = wl.make_config(3)
    dev = to_dev(torch, case)
    kinds = [(MUL, 0), (ADD, 0), (COMP, 0), (ADD, TRANSPOSED)]
    res = {k: run_gpu(torch, amla, case, dev, variant=k[0], flags=k[1] | BALANCED) for k in kinds}
    worst = {k: [0.0, 0.0] for k in kinds}
    for b in range(case.batch):
        want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens,
                                    case.softmax_scale, seq_ids=[b])
        for k, (out, lse) in res.items():
            assert np.all(np.abs(out[b] - want[b]) <= out_tolerance(want[b])), (b, k)
            worst[k][0] = max(worst[k][0], float(np.abs(out[b] - want[b]).max()))
            worst[k][1] = max(worst[k][1], float(np.abs(lse[b] - want_lse[b]).max()))
    for k in kinds:
        print(f"config 3 balanced {k}: max|out err| {worst[k][0]:.3e} max|lse err| {worst[k][1]:.3e}", flush=True)
        assert worst[k][1] <= LSE_TOL


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("workers", [0, 3, 11])
def test_causal_mask_among_the_query_tokens(env, kind, workers):
    """s_q = 4 under AMLA_FLAG_CAUSAL: tokens without any key (kv_len 1), limits at and just past block
    boundaries (whole blocks masked for the early tokens), 40 heads (two tokens per wave)."""
    torch, orc, amla, wl = env
    case = wl.make_case("causal", 44, batch=7, s_q=4, heads=40, seqlens=[1, 64, 0, 65, 66, 130, 300], spare_frac=0.25)
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale,
                                causal=True)
    out, lse = run_gpu(torch, amla, case, to_dev(torch, case), variant=kind[0], flags=kind[1] | CAUSAL,
                       num_splits=workers)
    check(out, lse, want, want_lse, f"causal workers={workers} {kind}")
    assert np.all(out[0, :3] == 0)


@pytest.mark.parametrize("kind,workers,causal", [((MUL, 0), 0, False), ((ADD, 0), 3, True), ((COMP, 0), 5, False),
                                                 ((ADD, 0), 9, False), ((MUL, TRANSPOSED), 0, False),
                                                 ((ADD, TRANSPOSED), 3, True), ((ADD, LAZY), 5, False), ((MUL, LAZY), 9, True)])
def test_per_sequence_query_counts(env, kind, workers, causal):
    """desc->q_lens: sequences with all, some, one and none of the s_q = 4 tokens, real and padding rows
    sharing a wave (40 heads), with and without the mask; padding rows come back as zeros / -inf."""
    torch, orc, amla, wl = env
    case = wl.make_case("qlens", 45, batch=7, s_q=4, heads=40, seqlens=[1, 64, 0, 65, 200, 130, 300], spare_frac=0.25)
    q_lens = np.array([4, 2, 3, 1, 0, 3, 4], np.int32)
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale,
                                causal=causal, q_lens=q_lens)
    out, lse = run_gpu(torch, amla, case, to_dev(torch, case), variant=kind[0],
                       flags=kind[1] | (CAUSAL if causal else BALANCED), num_splits=workers,
                       q_lens=torch.from_numpy(q_lens).cuda())
    check(out, lse, want, want_lse, f"q_lens workers={workers} causal={causal} {kind}")
    for b, k in enumerate(q_lens):
        assert np.all(out[b, k:] == 0) and np.all(np.isneginf(lse[b, k:]))


def test_causal_headline_shape_rows_match_shorter_caches(env):
    """At the headline shape (batch 128, s_q 2, 128 heads, kv 4096) the first token under the mask equals
    the unmasked run on caches one key shorter, the second token is unchanged."""
    torch, orc, amla, wl = env
    case = wl.make_config(2)
    dev = to_dev(torch, case)
    masked, masked_lse = run_gpu(torch, amla, case, dev, variant=ADD, flags=CAUSAL)
    plain, plain_lse = run_gpu(torch, amla, case, dev, variant=ADD, flags=BALANCED)
    q, kv, tab, lens = dev
    shorter, shorter_lse = amla.amla_decode(q, kv, tab, lens - 1, case.softmax_scale, variant=ADD, flags=BALANCED)
    torch.cuda.synchronize()
    shorter = shorter.float().cpu().numpy().astype(np.float64)
    assert np.array_equal(masked[:, 1], plain[:, 1]) and np.array_equal(masked_lse[:, 1], plain_lse[:, 1])
    assert np.array_equal(masked[:, 0], shorter[:, 0])
    assert np.abs(masked_lse[:, 0] - shorter_lse.cpu().numpy()[:, 0]).max() == 0
