"""The oracle's definition written a second time, in plain C with host pointers (oracle/amla_oracle_decode.c),
pinned the same way as the numpy form: against a pure-Python brute-force softmax, closed forms, and the numpy
form on ragged, paged, masked inputs; and its argument checks (it doubles as the host-side validator of block
ids and lengths)."""
import math

import numpy as np
import pytest

from oracle import amla_oracle as orc
from oracle import amla_oracle_c as orc_c
from paper_2509_25224_amd import workloads as wl


def _f32(x):
    """The C routine takes the scale as a float, like the library's entry point: both sides use that value."""
    return float(np.float32(x))


def _value(bits):
    return np.array([bits], dtype=np.uint16).astype(np.uint32).__lshift__(16).view(np.float32).astype(np.float64)[0]


def test_against_brute_force_in_pure_python():
    case = wl.make_case("brute_c", 91, batch=2, s_q=2, heads=3, seqlens=[70, 5], spare_frac=0.5)
    scale = _f32(case.softmax_scale)
    out, lse = orc_c.decode_c(case.q_bits, case.kv_bits, case.block_table, case.seqlens, scale)
    for b, L in enumerate(case.seqlens):
        rows = [[float(_value(x)) for x in case.kv_bits[case.block_table[b, j // 64], j % 64]] for j in range(L)]
        for t in range(2):
            for h in range(3):
                qv = [float(_value(x)) for x in case.q_bits[b, t, h]]
                s = [scale * math.fsum(a * c for a, c in zip(qv, r)) for r in rows]
                m = max(s)
                w = [math.exp(x - m) for x in s]
                Z = math.fsum(w)
                want = [math.fsum(w[j] * rows[j][d] for j in range(L)) / Z for d in range(512)]
                assert np.allclose(out[b, t, h], want, rtol=1e-12, atol=1e-14)
                assert abs(lse[b, t, h] - (m + math.log(Z))) < 1e-12


def test_closed_forms():
    # one key: the output is that key's value row exactly, lse its logit; no key: zeros and -inf
    case = wl.make_case("one_key_c", 92, batch=2, s_q=1, heads=4, seqlens=[1, 0])
    out, lse = orc_c.decode_c(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    row = orc.bf16_bits_to_f64(case.kv_bits[case.block_table[0, 0], 0])
    assert np.array_equal(out[0, 0], np.broadcast_to(row[:512], (4, 512)))
    q = orc.bf16_bits_to_f64(case.q_bits[0, 0])
    assert np.allclose(lse[0, 0], (q @ row) * _f32(case.softmax_scale), rtol=1e-13)
    assert np.all(out[1] == 0) and np.all(np.isneginf(lse[1]))
    # V is the first 512 columns, not the last
    assert not np.array_equal(row[:512], row[64:])
    # q = 0: uniform weights, out = mean of the value rows, lse = ln L
    flat = wl.make_case("flat_c", 93, batch=1, s_q=1, heads=2, seqlens=[100])
    flat.q_bits[:] = 0
    out, lse = orc_c.decode_c(flat.q_bits, flat.kv_bits, flat.block_table, flat.seqlens, flat.softmax_scale)
    K = orc.gather_kv(flat.kv_bits, flat.block_table[0], 100)
    assert np.allclose(out[0, 0, 0], K[:, :512].mean(axis=0), rtol=1e-12, atol=1e-15)
    assert np.allclose(lse, math.log(100.0))


@pytest.mark.parametrize("causal", [False, True])
def test_agrees_with_the_numpy_form(causal):
    case = wl.make_case("both", 94, batch=4, s_q=3, heads=5, seqlens=[129, 0, 64, 2], spare_frac=0.3, q_sigma=3.0)
    for q_lens in (None, [3, 1, 0, 2]):
        a, al = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, _f32(case.softmax_scale),
                           causal=causal, q_lens=q_lens)
        c, cl = orc_c.decode_c(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale,
                               causal=causal, q_lens=q_lens)
        assert np.allclose(a, c, rtol=1e-11, atol=1e-13)
        fin = np.isfinite(al)
        assert np.array_equal(al[~fin], cl[~fin]) and np.allclose(al[fin], cl[fin], rtol=1e-12, atol=1e-12)


def test_it_refuses_what_would_be_a_wild_read():
    case = wl.make_case("bad", 95, batch=2, s_q=1, heads=2, seqlens=[65, 10])
    args = (case.q_bits, case.kv_bits, None, None, case.softmax_scale)
    tab = case.block_table.copy()
    tab[0, 1] = case.num_blocks                               # a block id that is read and does not exist
    with pytest.raises(ValueError, match="-3"):
        orc_c.decode_c(args[0], args[1], tab, case.seqlens, args[4])
    tab = case.block_table.copy()
    tab[1, 1:] = -1                                           # entries past a sequence's last block are never read
    orc_c.decode_c(args[0], args[1], tab, case.seqlens, args[4])
    lens = case.seqlens.copy()
    lens[1] = 64 * case.block_table.shape[1] + 1
    with pytest.raises(ValueError, match="-2"):
        orc_c.decode_c(args[0], args[1], case.block_table, lens, args[4])
    with pytest.raises(ValueError, match="-4"):
        orc_c.decode_c(args[0], args[1], case.block_table, case.seqlens, args[4], q_lens=[1, 2])
