"""Planted mistakes: each plausible slip in the oracle's definition (a wrong slice, a dropped scale,
a wrong axis, a wrong sign, ignored paging ...) must make at least one of the pins fail.  The
mistakes are planted in the oracle on the CPU; nothing here touches the GPU path."""
import numpy as np
import pytest

from oracle import amla_oracle as orc
import test_oracle_definition as pins

PIN_TESTS = [
    lambda: pins.test_brute_force_tiny([70, 3], "random"),
    pins.test_torch_cpu_fp64_crosscheck,
    pins.test_zero_query_gives_mean_of_values_and_log_len,
    pins.test_single_key_returns_its_value_row_and_its_logit,
    pins.test_value_is_first_512_columns_not_last,
    pins.test_duplicated_keys_keep_out_and_add_ln2,
    pins.test_permuting_pages_with_table_changes_nothing,
    pins.test_partial_last_block_ignores_slots_past_the_end,
    pins.test_empty_sequence_convention,
    pins.test_scale_is_applied_to_logits,
]


def caught():
    for t in PIN_TESTS:
        try:
            t()
        except AssertionError:
            return True
        except Exception:          # a mutant may also crash a pin (shape errors): that counts as caught
            return True
    return False


def rows_mutant(kind):
    def f(Q, K, scale):
        G, L = Q.shape[0], K.shape[0]
        if L == 0:
            return np.zeros((G, 512)), np.full(G, -np.inf)
        V = K[:, 64:] if kind == "last_512" else K[:, :512]
        S = Q @ K.T if kind == "no_scale" else (Q @ K.T) * scale
        if kind == "reversed_k":
            S = (Q @ K[:, ::-1].T) * scale
        M = S.max(axis=1, keepdims=True)
        P = np.exp(M - S) if kind == "wrong_sign" else np.exp(S - M)
        axis = 0 if kind == "wrong_axis" else 1
        Z = P.sum(axis=axis, keepdims=True)
        out = P @ V if kind == "no_normalisation" else (P / Z) @ V if axis == 0 else (P @ V) / Z
        if kind == "lse_log2":
            lse = (M + np.log2(P.sum(axis=1, keepdims=True)))[:, 0]
        elif kind == "lse_without_max":
            lse = np.log(P.sum(axis=1))
        else:
            lse = (M + np.log(P.sum(axis=1, keepdims=True)))[:, 0]
        return out, lse
    return f


@pytest.mark.parametrize("kind", ["last_512", "no_scale", "reversed_k", "wrong_sign", "wrong_axis",
                                  "no_normalisation", "lse_log2", "lse_without_max"])
def test_mistake_in_attention_rows_is_caught(monkeypatch, kind):
    assert not caught()                                   # the real oracle passes every pin
    monkeypatch.setattr(orc, "attention_rows", rows_mutant(kind))
    assert caught(), kind


def test_ignoring_the_block_table_is_caught(monkeypatch):
    def gather(kv_bits, block_row, kv_len):
        nb = (kv_len + 63) // 64
        return orc.bf16_bits_to_f64(kv_bits[:nb].reshape(nb * 64, 576)[:kv_len])     # identity paging
    monkeypatch.setattr(orc, "gather_kv", gather)
    assert caught()


def test_reading_the_whole_last_block_is_caught(monkeypatch):
    def gather(kv_bits, block_row, kv_len):
        nb = (kv_len + 63) // 64
        pages = kv_bits[np.asarray(block_row[:nb], dtype=np.int64)]
        return orc.bf16_bits_to_f64(pages.reshape(nb * 64, 576))                      # no [:kv_len]
    monkeypatch.setattr(orc, "gather_kv", gather)
    assert caught()


def test_wrong_slot_order_inside_a_block_is_caught(monkeypatch):
    def gather(kv_bits, block_row, kv_len):
        nb = (kv_len + 63) // 64
        pages = kv_bits[np.asarray(block_row[:nb], dtype=np.int64)][:, ::-1]           # slots reversed
        return orc.bf16_bits_to_f64(pages.reshape(nb * 64, 576)[:kv_len])
    monkeypatch.setattr(orc, "gather_kv", gather)
    assert caught()


def test_wrong_exponent_shift_is_caught():
    """Lemma 3.1 with the mantissa width off by one (2^22 instead of 2^23) fails the worked example."""
    def bad_add(F, n):
        I = orc.as_int32(F).astype(np.int64) + np.asarray(n, dtype=np.int64) * (1 << 22)
        return orc.as_fp32(I.astype(np.int32))
    assert float(orc.exponent_add(np.float32(0.5), 1)) == 1.0
    assert float(bad_add(np.float32(0.5), 1)) != 1.0


def test_truncating_bf16_cast_is_caught_by_the_printed_accuracy_tables(monkeypatch):
    """Rounding P and the output to BF16 by truncation instead of round-to-nearest-even about doubles the
    error of both emulations; Table 3's N(0,1) column no longer comes out."""
    import test_oracle_method as method

    def truncate(x32):
        bits = np.asarray(x32, dtype=np.float32).view(np.uint32) & np.uint32(0xFFFF0000)
        return bits.view(np.float32)
    method.test_emulations_reproduce_the_printed_accuracy_tables("n", 1.0, 1.77e-3, 1.81e-3)
    monkeypatch.setattr(orc, "_round_bf16", truncate)
    with pytest.raises(AssertionError):
        method.test_emulations_reproduce_the_printed_accuracy_tables("n", 1.0, 1.77e-3, 1.81e-3)


def test_dropping_the_compensation_is_caught_by_the_printed_accuracy_tables(monkeypatch):
    """Algorithm 2 without its S32 / S16 / c_i / eps steps (S16 = 1, eps = 0: the weights 2^(t - m) S32 are rounded as
    they are) no longer reproduces the AMLA row of Table 3 on a peaked column."""
    import test_oracle_method as method

    def no_compensation(Q, K, V, scale, block=512, c_reading="appendix", guard=1e-6):
        out, _ = orc.amla_fp32_emulation(Q, K, V, scale, block=block)
        return out
    method.test_emulations_reproduce_the_printed_accuracy_tables("n", 4.0, 1.51e-3, 1.51e-3)
    monkeypatch.setattr(orc, "amla_alg2_emulation", no_compensation)
    with pytest.raises(AssertionError):
        method.test_emulations_reproduce_the_printed_accuracy_tables("n", 4.0, 1.51e-3, 1.51e-3)
