"""Seeded synthetic inputs for absorbed-MLA decode attention.

This module only *generates data*: bf16 bit patterns for the query tensor and the paged
latent KV pool, per-sequence lengths and block tables.  It contains none of the
attention arithmetic, so both the CPU oracle's tests and the HIP path's tests can draw
the same inputs from it without sharing any code of the method.

Tensors are numpy arrays on the host:
  q_bits       uint16 [batch, s_q, heads, 576]   bf16 bit patterns
  kv_bits      uint16 [num_blocks, 64, 576]      bf16 bit patterns (K = whole row,
                                                 V = first 512 columns of the same row)
  block_table  int32  [batch, max_blocks_per_seq] physical block of logical block j,
                                                 -1 where j is beyond the sequence
  seqlens      int32  [batch]

The recipe (shapes, N(0, sigma^2) values, permuted tables, lengths) follows the five
decode configurations this build is measured on; the paper's own experiments use the
same kind of synthetic Gaussian tensors and fixed shapes (Section 5.1 / 5.2).
"""
from __future__ import annotations

import dataclasses
import numpy as np

D_QK = 576          # latent 512 + RoPE 64  (Section 3.1: D_k = 576)
D_V = 512           # V is the first 512 columns of the cached row (D_v = 512)
BLOCK = 64          # keys per physical cache block
SOFTMAX_SCALE = 192.0 ** -0.5


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float32."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclasses.dataclass
class DecodeCase:
    name: str
    q_bits: np.ndarray
    kv_bits: np.ndarray
    block_table: np.ndarray
    seqlens: np.ndarray
    softmax_scale: float
    seed: int

    @property
    def batch(self) -> int:
        return int(self.q_bits.shape[0])

    @property
    def s_q(self) -> int:
        return int(self.q_bits.shape[1])

    @property
    def heads(self) -> int:
        return int(self.q_bits.shape[2])

    @property
    def num_blocks(self) -> int:
        return int(self.kv_bits.shape[0])

    @property
    def max_blocks_per_seq(self) -> int:
        return int(self.block_table.shape[1])

    @property
    def total_kv(self) -> int:
        return int(self.seqlens.astype(np.int64).sum())


def _rng(seed: int, stream: int) -> np.random.Generator:
    # Philox is counter based: (seed, stream) selects an independent, reproducible stream.
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(stream)]))


def _normal_bf16(rng: np.random.Generator, shape, sigma: float, dist: str = "normal") -> np.ndarray:
    """dist = "normal": N(0, sigma^2); dist = "uniform": U(-sigma, sigma).  Drawn in FP32, rounded to bf16."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24                      # bounded temporary memory for the big pools
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        if dist == "normal":
            x = rng.standard_normal(hi - lo, dtype=np.float32)
        elif dist == "uniform":
            x = rng.random(hi - lo, dtype=np.float32) * np.float32(2) - np.float32(1)
        else:
            raise ValueError(dist)
        if sigma != 1.0:
            x *= np.float32(sigma)
        out[lo:hi] = f32_to_bf16_bits(x)
    return out.reshape(shape)


def make_case(name: str, seed: int, batch: int, s_q: int, heads: int, seqlens,
              q_sigma: float = 1.0, kv_sigma: float = 1.0, table: str = "random",
              spare_frac: float = 0.0, softmax_scale: float = SOFTMAX_SCALE,
              max_blocks_per_seq: int | None = None, dist: str = "normal") -> DecodeCase:
    """Build one decode problem.

    dist = "normal": q ~ N(0, q_sigma^2), cache ~ N(0, kv_sigma^2); dist = "uniform": U(-q_sigma, q_sigma)
    and U(-kv_sigma, kv_sigma).

    table = "identity": sequence b owns consecutive physical blocks in order.
    table = "random"  : the physical blocks are a random permutation dealt to the
                        sequences (non-contiguous, out of order); `spare_frac` adds
                        unused blocks (also filled with finite data) to the pool.
    Every slot of the pool holds a finite value, including slots past a sequence's end
    inside its last block.
    """
    seqlens = np.asarray(seqlens, dtype=np.int32).reshape(batch)
    nb = (seqlens.astype(np.int64) + BLOCK - 1) // BLOCK
    need = int(nb.sum())
    num_blocks = max(1, need + int(np.ceil(need * spare_frac)))
    mbs = int(max(1, nb.max() if batch else 1))
    if max_blocks_per_seq is not None:
        assert max_blocks_per_seq >= mbs
        mbs = int(max_blocks_per_seq)

    q_bits = _normal_bf16(_rng(seed, 0), (batch, s_q, heads, D_QK), q_sigma, dist)
    kv_bits = _normal_bf16(_rng(seed, 1), (num_blocks, BLOCK, D_QK), kv_sigma, dist)

    if table == "identity":
        phys = np.arange(num_blocks, dtype=np.int32)
    elif table == "random":
        phys = _rng(seed, 3).permutation(num_blocks).astype(np.int32)
    else:
        raise ValueError(table)
    block_table = np.full((batch, mbs), -1, dtype=np.int32)
    at = 0
    for b in range(batch):
        k = int(nb[b])
        block_table[b, :k] = phys[at:at + k]
        at += k
    return DecodeCase(name, q_bits, kv_bits, block_table, seqlens, float(softmax_scale), seed)


def ragged_lengths(seed: int, batch: int, lo: int, hi: int) -> np.ndarray:
    """kv_len per sequence, uniform integers in [lo, hi]."""
    return _rng(seed, 2).integers(lo, hi + 1, size=batch, dtype=np.int64).astype(np.int32)


# The five measured configurations: (name, seed, batch, s_q, heads, lengths, q_sigma, table)
CONFIG_NAMES = ("tiny", "decode_b64", "mtp_b128", "ragged_b32", "long_b8")


def make_config(index: int) -> DecodeCase:
    """configs[index] of the measured workloads (0-based)."""
    if index == 0:
        return make_case("tiny", 0, 1, 1, 16, [256], table="identity")
    if index == 1:
        return make_case("decode_b64", 1, 64, 1, 128, [4096] * 64)
    if index == 2:
        return make_case("mtp_b128", 2, 128, 2, 128, [4096] * 128)
    if index == 3:
        lens = ragged_lengths(3, 32, 1024, 16384)
        return make_case("ragged_b32", 3, 32, 2, 128, lens, spare_frac=0.125)
    if index == 4:
        return make_case("long_b8", 4, 8, 4, 128, [65536] * 8, q_sigma=4.0)
    raise IndexError(index)


def make_low_head_case(heads: int = 16, batch: int = 256, kv_len: int = 4096, seed: int = 7) -> DecodeCase:
    """A low-head-count decode batch: what one GPU of a tensor-parallel group sees of the 128-head model (16
    heads at eight-way sharding), s_q = 1, every sequence kv_len long, random block table.  With 16 rows per
    cached row the shape has 30 FLOP per byte and is bound by HBM."""
    return make_case(f"low_heads_h{heads}_b{batch}", seed, batch, 1, heads, [kv_len] * batch)


def make_table5_case(s_q: int, s_k: int, seed: int = 5) -> DecodeCase:
    """A shape of the paper's performance table (Section 5.2, Table 5): batch 96, 128 query heads on
    one shared KV head, BF16, every sequence s_k long, s_q in {1, 2}, cache laid out contiguously
    (identity block table)."""
    return make_case(f"table5_sq{s_q}_sk{s_k}", seed, 96, s_q, 128, [s_k] * 96, table="identity")


def make_accuracy_case(family: str, param: float, seed: int = 6, batch: int = 2, heads: int = 128) -> DecodeCase:
    """An input of the paper's accuracy experiment (Section 5.1, Tables 3 and 4): Q and the cache drawn
    from N(0, param^2) (family "n") or U(-param, param) (family "u"), context length 8K, BF16, V the
    first 512 columns of the cached row, softmax scale 1 / sqrt(576) (Eq. (1) with D_k = 576; the
    setting under which FP32 emulations of Algorithms 1 and 2 reproduce the printed errors)."""
    dist = {"n": "normal", "u": "uniform"}[family]
    return make_case(f"accuracy_{family}{param:g}", seed, batch, 1, heads, [8192] * batch, q_sigma=param,
                     kv_sigma=param, softmax_scale=D_QK ** -0.5, dist=dist)
