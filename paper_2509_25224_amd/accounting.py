"""FLOP and byte accounting for decode attention (Section 2.4, arithmetic intensity).

FLOPS = 2 * N1 * S1 * S2 * (D_k + D_v) per sequence; KV bytes for MLA = 2 * S2 * D_k
(one bf16 latent row per cached token, shared by every head); for MHA/GQA
2 * N2 * S2 * (D_k + D_v).  Only useful work is counted: no masked tail keys, padding
rows or split-combine work.
"""
from __future__ import annotations


def decode_flops(heads: int, s_q: int, total_kv: int, d_qk: int = 576, d_v: int = 512) -> int:
    return 2 * heads * s_q * total_kv * (d_qk + d_v)


def kv_bytes_mla(total_kv: int, d_qk: int = 576, elem: int = 2) -> int:
    return elem * total_kv * d_qk


def kv_bytes_mha_gqa(kv_heads: int, total_kv: int, d_qk: int, d_v: int, elem: int = 2) -> int:
    return elem * kv_heads * total_kv * (d_qk + d_v)


def algorithmic_bytes(heads: int, s_q: int, batch: int, total_kv: int,
                      d_qk: int = 576, d_v: int = 512) -> int:
    """KV rows read once + q read once + bf16 out and f32 lse written once."""
    rows = batch * s_q * heads
    return kv_bytes_mla(total_kv, d_qk) + rows * (2 * d_qk + 2 * d_v + 4)
