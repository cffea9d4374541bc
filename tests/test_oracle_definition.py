"""Pins for the oracle's attention definition (Eq. (1), Section 2.2 shapes) and for the
paged / ragged conventions.  None of these call the oracle to produce their expected
values: they use pure-Python brute force, torch's CPU fp64 routines, or closed forms."""
import math

import numpy as np
import pytest
import torch

from oracle import amla_oracle as orc
from paper_2509_25224_amd import workloads as wl


def _bf16_val(bits: int) -> float:
    import struct
    return struct.unpack("<f", struct.pack("<I", int(bits) << 16))[0]


def _brute_force(case, b, t, h):
    """Direct exp(s_j) / sum exp(s_k) with Python floats, no max subtraction, explicit
    page lookup.  Valid for the small logits of the tiny cases used here."""
    L = int(case.seqlens[b])
    q = [_bf16_val(x) for x in case.q_bits[b, t, h]]
    w = []
    rows = []
    for j in range(L):
        page = int(case.block_table[b, j // 64])
        row = [_bf16_val(x) for x in case.kv_bits[page, j % 64]]
        s = case.softmax_scale * math.fsum(qd * kd for qd, kd in zip(q, row))
        w.append(math.exp(s))
        rows.append(row)
    Z = math.fsum(w)
    out = [math.fsum(w[j] * rows[j][d] for j in range(L)) / Z for d in range(512)]
    return out, math.log(Z)


@pytest.mark.parametrize("lens,table", [([5], "identity"), ([70, 3], "random"), ([64, 65], "random")])
def test_brute_force_tiny(lens, table):
    case = wl.make_case("t", 11, len(lens), 2, 2, lens, table=table)
    out, lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    for b in range(case.batch):
        for t in range(2):
            for h in range(2):
                eo, el = _brute_force(case, b, t, h)
                assert np.allclose(out[b, t, h], eo, rtol=0, atol=1e-12)
                assert abs(lse[b, t, h] - el) < 1e-12


def test_torch_cpu_fp64_crosscheck():
    """Library-routine cross-check on config-1-sized input: torch.softmax / matmul in fp64
    over keys gathered with torch indexing."""
    case = wl.make_config(0)
    out, lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    kv = torch.from_numpy(wl.bf16_bits_to_f32(case.kv_bits)).double()
    q = torch.from_numpy(wl.bf16_bits_to_f32(case.q_bits)).double()
    for b in range(case.batch):
        L = int(case.seqlens[b])
        pages = torch.from_numpy(case.block_table[b, : (L + 63) // 64].astype(np.int64))
        K = kv[pages].reshape(-1, 576)[:L]
        S = torch.einsum("thd,ld->thl", q[b], K) * case.softmax_scale
        eo = torch.einsum("thl,ld->thd", torch.softmax(S, dim=-1), K[:, :512])
        el = torch.logsumexp(S, dim=-1)
        assert np.abs(out[b] - eo.numpy()).max() < 1e-12
        assert np.abs(lse[b] - el.numpy()).max() < 1e-12


def test_zero_query_gives_mean_of_values_and_log_len():
    case = wl.make_case("z", 5, 2, 1, 4, [200, 64])
    case.q_bits[...] = 0
    out, lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    for b in range(2):
        L = int(case.seqlens[b])
        V = np.stack([wl.bf16_bits_to_f32(case.kv_bits[case.block_table[b, j // 64], j % 64, :512]).astype(np.float64)
                      for j in range(L)])
        assert np.abs(out[b, 0] - V.mean(axis=0)).max() < 1e-13
        assert np.abs(lse[b] - math.log(L)).max() < 1e-13


def test_single_key_returns_its_value_row_and_its_logit():
    case = wl.make_case("one", 6, 1, 1, 3, [1])
    out, lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    row = wl.bf16_bits_to_f32(case.kv_bits[case.block_table[0, 0], 0]).astype(np.float64)
    q = wl.bf16_bits_to_f32(case.q_bits[0, 0]).astype(np.float64)
    assert np.array_equal(out[0, 0], np.broadcast_to(row[:512], (3, 512)))
    assert np.allclose(lse[0, 0], case.softmax_scale * (q @ row), rtol=0, atol=1e-13)


def test_value_is_first_512_columns_not_last():
    """A wrong V slice (e.g. the last 512 columns) must show: make the two slices differ
    by construction and check against the L = 1 closed form per column."""
    case = wl.make_case("slice", 7, 1, 1, 2, [1])
    out, _ = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    row = wl.bf16_bits_to_f32(case.kv_bits[case.block_table[0, 0], 0]).astype(np.float64)
    assert not np.array_equal(row[:512], row[64:])
    assert np.array_equal(out[0, 0, 0], row[:512])


def test_duplicated_keys_keep_out_and_add_ln2():
    base = wl.make_case("d1", 8, 1, 2, 4, [128], table="identity")
    dup_kv = np.concatenate([base.kv_bits, base.kv_bits], axis=0)
    table = np.arange(4, dtype=np.int32).reshape(1, 4)
    o1, l1 = orc.decode(base.q_bits, base.kv_bits, base.block_table, base.seqlens, base.softmax_scale)
    o2, l2 = orc.decode(base.q_bits, dup_kv, table, np.array([256], np.int32), base.softmax_scale)
    assert np.abs(o1 - o2).max() < 1e-13
    assert np.abs(l2 - l1 - math.log(2)).max() < 1e-13


def test_permuting_pages_with_table_changes_nothing():
    case = wl.make_case("p", 9, 2, 1, 4, [300, 130], table="identity")
    o1, l1 = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    perm = np.random.default_rng(0).permutation(case.num_blocks)
    kv2 = np.empty_like(case.kv_bits)
    kv2[perm] = case.kv_bits                     # old block i now lives at perm[i]
    tab2 = np.where(case.block_table >= 0, perm[np.maximum(case.block_table, 0)], -1).astype(np.int32)
    o2, l2 = orc.decode(case.q_bits, kv2, tab2, case.seqlens, case.softmax_scale)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


def test_partial_last_block_ignores_slots_past_the_end():
    case = wl.make_case("tail", 10, 1, 1, 2, [70])
    o1, l1 = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    kv2 = case.kv_bits.copy()
    kv2[case.block_table[0, 1], 6:] = wl.f32_to_bf16_bits(np.full((58, 576), 77.0, np.float32))
    o2, l2 = orc.decode(case.q_bits, kv2, case.block_table, case.seqlens, case.softmax_scale)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


def test_empty_sequence_convention():
    case = wl.make_case("e", 12, 2, 1, 2, [0, 10])
    out, lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    assert np.all(out[0] == 0) and np.all(np.isneginf(lse[0]))
    assert np.all(np.isfinite(out[1])) and np.all(np.isfinite(lse[1]))


def test_s_q_tokens_are_independent_rows_without_mask():
    """Each of the s_q query tokens sees the whole cached prefix: token t's rows equal a
    one-token problem built from that token alone."""
    case = wl.make_case("mtp", 13, 1, 3, 2, [100])
    out, lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    for t in range(3):
        o1, l1 = orc.decode(case.q_bits[:, t:t + 1], case.kv_bits, case.block_table, case.seqlens,
                            case.softmax_scale)
        assert np.array_equal(out[:, t], o1[:, 0]) and np.array_equal(lse[:, t], l1[:, 0])


def test_scale_is_applied_to_logits():
    """scale -> 0 must approach the uniform average; a dropped scale would not."""
    case = wl.make_case("sc", 14, 1, 1, 2, [50])
    out, lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, 0.0)
    V = orc.gather_kv(case.kv_bits, case.block_table[0], 50)[:, :512]
    assert np.abs(out[0, 0] - V.mean(axis=0)).max() < 1e-13
    assert np.abs(lse - math.log(50)).max() < 1e-13


def test_workload_shapes_of_the_tiny_config():
    case = wl.make_config(0)
    assert case.q_bits.shape == (1, 1, 16, 576)
    assert case.kv_bits.shape == (4, 64, 576)
    assert case.block_table.tolist() == [[0, 1, 2, 3]]
    assert case.seqlens.tolist() == [256]
    assert abs(case.softmax_scale - 192 ** -0.5) < 1e-15


def test_bf16_rounding_of_generator_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.140625], np.float32)
    # 1 + 2^-8 is a tie between 1.0 and 1+2^-7 -> even (1.0); 1 + 3*2^-8 ties up to 1+2^-6
    bits = wl.f32_to_bf16_bits(x)
    back = wl.bf16_bits_to_f32(bits)
    assert back.tolist() == [1.0, 1.0, 1.015625, -2.5, 3.140625]


# ------------------------------------------------------------------ causal mask among the s_q tokens
def test_causal_rows_equal_unmasked_rows_of_a_shorter_cache():
    """Token t of s_q under the causal mask is, by definition, the unmasked single-token problem on the
    first kv_len - (s_q - 1 - t) keys; the last token sees everything, and with s_q = 1 the mask
    changes nothing.  A token with no key gets the empty-sequence convention."""
    case = wl.make_case("causal", 61, batch=3, s_q=3, heads=4, seqlens=[1, 66, 130], spare_frac=0.3)
    masked, masked_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale,
                                    causal=True)
    plain, plain_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    assert np.array_equal(masked[:, 2], plain[:, 2]) and np.array_equal(masked_lse[:, 2], plain_lse[:, 2])
    for t in range(3):
        shorter = np.maximum(case.seqlens - (2 - t), 0).astype(np.int32)
        one, one_lse = orc.decode(case.q_bits[:, t:t + 1], case.kv_bits, case.block_table, shorter, case.softmax_scale)
        assert np.array_equal(masked[:, t], one[:, 0]) and np.array_equal(masked_lse[:, t], one_lse[:, 0])
    # kv_len 1: tokens 0 and 1 have no key at all
    assert np.all(masked[0, :2] == 0) and np.all(np.isneginf(masked_lse[0, :2]))
    single = wl.make_case("causal1", 62, batch=2, s_q=1, heads=4, seqlens=[5, 70])
    a = orc.decode(single.q_bits, single.kv_bits, single.block_table, single.seqlens, single.softmax_scale, causal=True)
    b = orc.decode(single.q_bits, single.kv_bits, single.block_table, single.seqlens, single.softmax_scale)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_causal_mask_against_brute_force():
    """Pure-Python softmax with the mask written out key by key."""
    import math
    case = wl.make_case("causal_bf", 63, batch=1, s_q=2, heads=2, seqlens=[5], table="identity")
    got, got_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale, causal=True)
    q = wl.bf16_bits_to_f32(case.q_bits).astype(float)
    kv = wl.bf16_bits_to_f32(case.kv_bits).astype(float)[0]
    for t in range(2):
        for h in range(2):
            visible = [j for j in range(5) if j <= 5 - 2 + t]          # keys 0 .. kv_len - s_q + t
            logits = [case.softmax_scale * sum(q[0, t, h, d] * kv[j, d] for d in range(576)) for j in visible]
            z = sum(math.exp(x) for x in logits)
            for d in (0, 17, 511):
                want = sum(math.exp(x) / z * kv[j, d] for x, j in zip(logits, visible))
                assert abs(got[0, t, h, d] - want) < 1e-12
            assert abs(got_lse[0, t, h] - math.log(z)) < 1e-12


# ------------------------------------------------------------------ per-sequence number of query tokens
@pytest.mark.parametrize("causal", [False, True])
def test_q_lens_is_the_smaller_problem_on_the_first_tokens(causal):
    """A sequence with q_lens[b] = k is, by definition, the s_q = k problem on its first k tokens; the
    padding tokens get the empty convention; q_lens = s_q everywhere is the plain problem."""
    case = wl.make_case("qlens", 64, batch=4, s_q=3, heads=4, seqlens=[130, 66, 5, 70], spare_frac=0.3)
    q_lens = np.array([3, 1, 2, 0], np.int32)
    got, got_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale,
                              causal=causal, q_lens=q_lens)
    for b, k in enumerate(q_lens):
        assert np.all(got[b, k:] == 0) and np.all(np.isneginf(got_lse[b, k:]))
        if k:
            want, want_lse = orc.decode(case.q_bits[:, :k], case.kv_bits, case.block_table, case.seqlens,
                                        case.softmax_scale, seq_ids=[b], causal=causal)
            assert np.array_equal(got[b, :k], want[b]) and np.array_equal(got_lse[b, :k], want_lse[b])
    full = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale, causal=causal,
                      q_lens=np.full(4, 3, np.int32))
    plain = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale, causal=causal)
    assert np.array_equal(full[0], plain[0]) and np.array_equal(full[1], plain[1])


def test_q_lens_with_the_mask_against_brute_force():
    """Two of three tokens present, mask written out key by key: token t of k sees keys 0 .. kv_len - k + t."""
    import math
    case = wl.make_case("qlens_bf", 65, batch=1, s_q=3, heads=2, seqlens=[6], table="identity")
    got, got_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale,
                              causal=True, q_lens=[2])
    q = wl.bf16_bits_to_f32(case.q_bits).astype(float)
    kv = wl.bf16_bits_to_f32(case.kv_bits).astype(float)[0]
    for t in range(2):
        for h in range(2):
            visible = [j for j in range(6) if j <= 6 - 2 + t]
            logits = [case.softmax_scale * sum(q[0, t, h, d] * kv[j, d] for d in range(576)) for j in visible]
            z = sum(math.exp(x) for x in logits)
            for d in (0, 300, 511):
                want = sum(math.exp(x) / z * kv[j, d] for x, j in zip(logits, visible))
                assert abs(got[0, t, h, d] - want) < 1e-12
            assert abs(got_lse[0, t, h] - math.log(z)) < 1e-12
    assert np.all(got[0, 2] == 0) and np.all(np.isneginf(got_lse[0, 2]))
