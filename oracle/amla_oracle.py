"""CPU oracle for absorbed-MLA decode attention.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain reference the HIP kernels are checked against.  It shares no
code with the GPU path and must never be imported by the product (the package under
`paper_2509_25224_amd/`); only tests, the smoke check and the benchmark's CPU-baseline
leg call it.

What it holds
-------------
* `decode`             the *definition* of the result: Eq. (1) softmax(Q K^T * scale) V in
                       fp64 over the exact values of the bf16 inputs, with K the 576-wide
                       cached row and V its first 512 columns (Section 2.2, Section 3.1),
                       two-pass safe softmax, plus lse = max + ln(sum).  The paper's
                       "Golden" (Section 5.1) in fp64 instead of fp32.  Options outside the paper:
                       a causal mask among the s_q tokens and per-sequence query counts.
                       (`amla_oracle_decode.c` beside this file is the same definition as plain C loops
                       with host pointers, in the argument order of the library's entry point; it is
                       pinned on its own and against this function by tests/test_oracle_c.py.)
* `flash_attention`    Algorithm 1 (FlashAttention / "Base") written step by step in fp64.
* `amla_recurrence`    Eq. (4): the AMLA transform with n_i = round(-m_i / ln 2) and
                       r_i = exp(-n_i ln 2 - m_i), in fp64.
* `as_int32`/`as_fp32`/`exponent_add`           Eq. (5)-(8), Lemma 3.1 on FP32 bit patterns.
* `exponent_add_guarded`                        the wrap-safe reading of Lemma 3.1's range
                                                condition (see below).
* `amla_fp32_emulation` Algorithm 2's loop in FP32 with BF16 P and the INT32 exponent add,
                       without the BF16 scale compensation (the S32 / S16 / c_i steps).
* `flash_fp32_emulation` Algorithm 1 in FP32 with BF16 P (the paper's "Base", Section 5.1).
* `amla_comp_fp32_emulation` Algorithm 2 with its BF16 scale compensation (Appendix A) in base 2 with one
                       reference per row; defaults = the form of the kernels' ADD_COMP variant, options
                       for either definition of c_i, the truncating cast with its guard, the plain add
                       and the FP32 normaliser.
* `amla_alg2_emulation` the same with the paper's own parameter choices (512-key blocks, truncating
                       cast with 1e-6, plain add, FP32 row sum).
* `frobenius_error`    the error metric of Section 5.1.

Pins (tests/test_oracle_*.py): the worked example of Section 3.2 (0.5 <-> 126 * 2^23),
Lemma 3.1 against ldexp, brute-force softmax in pure Python, torch CPU fp64, closed forms
(q = 0, one key, duplicated keys, permuted pages), chunk-size and chunk-order invariance
of Algorithm 1, Eq. (4) == Eq. (2), 1/sqrt2 <= r_i <= sqrt2, Table 2 and Table 5
arithmetic.  Paging, ragged lengths and LSE are not in the paper; their conventions are
pinned by the closed forms and the metamorphic (permutation / duplication) tests only.

Readings taken where the paper is silent
----------------------------------------
* scale: the paper divides by sqrt(D_k); here the caller passes `softmax_scale`.
* round(): round-half-even.  Any integer within 1/2 of -m/ln2 keeps r in [1/sqrt2, sqrt2].
* first block: no rescale (n_0 = -inf, "if i > 1" in Algorithm 2).
* empty sequence (kv_len 0): out = 0, lse = -inf.
* exponent add outside Lemma 3.1's range: E + n < 0 (including F = +-0 with n < 0) gives a
  zero with F's sign, E + n == 0 gives the mantissa bits alone (magnitude < 2^-126); never
  the wrapped bit pattern.
"""
from __future__ import annotations

import math
import numpy as np

D_QK = 576
D_V = 512
BLOCK = 64
LN2 = math.log(2.0)


# --------------------------------------------------------------------------------------
# bf16 bit patterns -> exact real values
# --------------------------------------------------------------------------------------
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def gather_kv(kv_bits: np.ndarray, block_row: np.ndarray, kv_len: int) -> np.ndarray:
    """Logical key j of a sequence lives in physical block block_row[j // 64], slot j % 64."""
    nb = (kv_len + BLOCK - 1) // BLOCK
    pages = kv_bits[np.asarray(block_row[:nb], dtype=np.int64)]        # [nb, 64, 576]
    return bf16_bits_to_f64(pages.reshape(nb * BLOCK, D_QK)[:kv_len])


# --------------------------------------------------------------------------------------
# The definition (Eq. (1)) -- what every variant of the kernel must reproduce
# --------------------------------------------------------------------------------------
def attention_rows(Q: np.ndarray, K: np.ndarray, scale: float):
    """softmax(scale * Q K^T) V with V = K[:, :512]; Q [G,576], K [L,576], all fp64.

    Returns (out [G,512], lse [G]).  Two passes: row max first, then exp and sums.
    """
    G = Q.shape[0]
    L = K.shape[0]
    if L == 0:
        return np.zeros((G, D_V)), np.full(G, -np.inf)
    S = (Q @ K.T) * scale                      # [G, L]
    M = S.max(axis=1, keepdims=True)
    P = np.exp(S - M)
    Z = P.sum(axis=1, keepdims=True)
    out = (P @ K[:, :D_V]) / Z
    lse = (M + np.log(Z))[:, 0]
    return out, lse


def decode(q_bits, kv_bits, block_table, seqlens, softmax_scale, seq_ids=None, causal=False, q_lens=None):
    """Decode attention for every row (b, t, h).  Without `causal` all s_q query tokens of a
    sequence see all kv_len cached keys (no mask among them).  With `causal` the s_q tokens are the
    last s_q positions of the cache and token t sees keys 0 .. kv_len - s_q + t, that is the first
    kv_len - (s_q - 1 - t) keys (none if that is <= 0: out = 0, lse = -inf).  The paper has no mask
    (its kernel is quoted for s_q in {1, 2} without one); this is the usual multi-token-prediction
    convention.  `q_lens` (int [B], 0 <= q_lens[b] <= s_q) gives every sequence its own number of query
    tokens in the padded q array: sequence b is the problem with s_q = q_lens[b] on its first q_lens[b]
    tokens, and the rows of the padding tokens are out = 0, lse = -inf (a convention of this library;
    the paper's kernel has one s_q for the batch).

    q_bits uint16 [B,T,H,576]; kv_bits uint16 [nblk,64,576]; block_table int32 [B,maxb];
    seqlens int32 [B].  Returns out float64 [B,T,H,512] (not rounded), lse float64 [B,T,H].
    `seq_ids` restricts the work to some sequences (others are left as NaN).
    """
    B, T, H, D = q_bits.shape
    assert D == D_QK and kv_bits.shape[1:] == (BLOCK, D_QK)
    out = np.full((B, T, H, D_V), np.nan)
    lse = np.full((B, T, H), np.nan)
    for b in (range(B) if seq_ids is None else seq_ids):
        L = int(seqlens[b])
        K = gather_kv(kv_bits, block_table[b], L)
        Tb = T if q_lens is None else int(q_lens[b])
        assert 0 <= Tb <= T
        out[b, Tb:] = 0.0
        lse[b, Tb:] = -np.inf
        if not causal:
            Q = bf16_bits_to_f64(q_bits[b, :Tb]).reshape(Tb * H, D_QK)
            o, l = attention_rows(Q, K, float(softmax_scale))
            out[b, :Tb] = o.reshape(Tb, H, D_V)
            lse[b, :Tb] = l.reshape(Tb, H)
        else:
            for t in range(Tb):
                limit = max(L - (Tb - 1 - t), 0)
                out[b, t], lse[b, t] = attention_rows(bf16_bits_to_f64(q_bits[b, t]), K[:limit], float(softmax_scale))
    return out, lse


# --------------------------------------------------------------------------------------
# Algorithm 1 (FlashAttention, "Base"), fp64
# --------------------------------------------------------------------------------------
def flash_attention(Q, K, V, scale, blocks):
    """`blocks` is a list of index arrays partitioning range(len(K)); they are visited in
    the given order.  Returns (O, m_N, l_N) with O already divided by l_N."""
    G = Q.shape[0]
    O = np.zeros((G, V.shape[1]))
    m = np.full((G, 1), -np.inf)
    l = np.zeros((G, 1))
    for idx in blocks:
        S = (Q @ K[idx].T) * scale                                   # [C1]
        m_new = np.maximum(m, S.max(axis=1, keepdims=True))          # [V1]
        P = np.exp(S - m_new)
        alpha = np.exp(m - m_new)
        l = l * alpha + P.sum(axis=1, keepdims=True)
        T = P @ V[idx]                                               # [C2]
        O = O * alpha + T                                            # [V2]
        m = m_new
    return O / l, m[:, 0], l[:, 0]


# --------------------------------------------------------------------------------------
# Eq. (4): AMLA recurrence, fp64
# --------------------------------------------------------------------------------------
def amla_recurrence(Q, K, V, scale, blocks):
    """O~_i = O~_{i-1} * 2^(n_i - n_{i-1}) + (1/r_i) P_i V_i, with O~_i = O_i / r_i.

    Returns (O, r_trace) where O = O~_N * r_N / l_N is the attention output and r_trace
    lists every r_i that occurred (all rows, all blocks).
    """
    G = Q.shape[0]
    Ot = np.zeros((G, V.shape[1]))
    m = np.full((G, 1), -np.inf)
    l = np.zeros((G, 1))
    n = None
    r = None
    r_trace = []
    for idx in blocks:
        S = (Q @ K[idx].T) * scale
        m_new = np.maximum(m, S.max(axis=1, keepdims=True))
        P = np.exp(S - m_new)
        l = l * np.exp(m - m_new) + P.sum(axis=1, keepdims=True)
        n_new = np.rint(-m_new / LN2)
        r = np.exp(-n_new * LN2 - m_new)
        r_trace.append(r.copy())
        if n is not None:                       # first block: accumulator is zero
            Ot = Ot * np.exp2(n_new - n)
        Ot = Ot + (P @ V[idx]) / r
        m, n = m_new, n_new
    return Ot * r / l, np.concatenate(r_trace)


# --------------------------------------------------------------------------------------
# FP32 <-> INT32 (Eq. (5)-(8), Lemma 3.1)
# --------------------------------------------------------------------------------------
def as_int32(f) -> np.ndarray:
    return np.asarray(f, dtype=np.float32).view(np.int32)


def as_fp32(i) -> np.ndarray:
    return np.asarray(i, dtype=np.int32).view(np.float32)


def exponent_add(F, n) -> np.ndarray:
    """AS_FP32(AS_INT32(F) + n * 2^23), two's-complement wrap-around like the hardware."""
    I = as_int32(F).astype(np.int64)
    s = I + np.asarray(n, dtype=np.int64) * (1 << 23)
    s = ((s + (1 << 31)) % (1 << 32)) - (1 << 31)
    return as_fp32(s.astype(np.int32))


def exponent_add_guarded(F, n) -> np.ndarray:
    """Exponent add for n <= 0 that never wraps: where the biased exponent E of F has
    E + n < 0 the result is a zero carrying F's sign.  E + n == 0 leaves the exponent
    field empty and the mantissa bits in place: a value of magnitude < 2^-126 (the paper
    neglects subnormals, Section 3.2; any |result| <= 2^-126 is as good as zero here)."""
    F = np.asarray(F, dtype=np.float32)
    n = np.asarray(n, dtype=np.int64)
    assert np.all(n <= 0)
    I = as_int32(F).astype(np.int64)
    E = (I >> 23) & 0xFF
    ok = (E + n) >= 0
    raw = exponent_add(F, n)
    zero = as_fp32((as_int32(F) & np.int32(-2**31)))
    return np.where(ok, raw, zero)


# --------------------------------------------------------------------------------------
# Algorithm 2's loop in FP32 with BF16 P and INT32 exponent add (no BF16 scale
# compensation: its S32 / S16 / c_i steps with S16 := S32, c_i := 1, eps := 0)
# --------------------------------------------------------------------------------------
def _round_bf16(x32: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def amla_fp32_emulation(Q, K, V, scale, block=64, clamp=-30, lazy_threshold=None, normalise="f32"):
    """Q, K, V are float32 arrays holding bf16-exact values.  Uses base-2 exponentials
    (t = s * scale * log2 e), mu_i = rint(max t) (= -n_i), P = 2^(t - mu_i) rounded to BF16
    for the PV product, FP32 row sum for l, exponent add for the rescale.  With
    `lazy_threshold` the reference mu is only moved when the row max exceeds it by more than
    that many base-2 units (the weights may then grow up to 2^threshold).  `normalise` chooses
    what divides the accumulator at the end: "f32", the FP32 sum of the unrounded weights (as
    Algorithm 2 sums them), or "b16", a second row sum over the BF16-rounded weights that
    entered the product (lse always comes from the FP32 sum)."""
    f32 = np.float32
    G, L = Q.shape[0], K.shape[0]
    O = np.zeros((G, V.shape[1]), dtype=f32)
    l = np.zeros(G, dtype=f32)
    l16 = np.zeros(G, dtype=f32)
    m = np.full(G, -np.inf, dtype=f32)
    mu = None
    c = f32(scale * math.log2(math.e))
    for lo in range(0, L, block):
        Kb, Vb = K[lo:lo + block], V[lo:lo + block]
        t = (Q @ Kb.T).astype(f32) * c
        m = np.maximum(m, t.max(axis=1))
        mu_new = np.rint(m)
        if lazy_threshold is not None and mu is not None:
            mu_new = np.where(m > mu + lazy_threshold, mu_new, mu)
        P = np.exp2((t - mu_new[:, None]).astype(f32)).astype(f32)
        Pb = _round_bf16(P)
        if mu is not None:
            d = np.maximum(mu - mu_new, clamp).astype(np.int64)      # <= 0
            O = exponent_add_guarded(O, d[:, None])
            l = exponent_add_guarded(l, d)
            l16 = exponent_add_guarded(l16, d)
        l = (l + P.sum(axis=1, dtype=f32)).astype(f32)
        l16 = (l16 + Pb.sum(axis=1, dtype=f32)).astype(f32)
        O = (O + (Pb @ Vb).astype(f32)).astype(f32)
        mu = mu_new
    out = O / (l16 if normalise == "b16" else l)[:, None]
    lse = (mu.astype(np.float64) + np.log2(l.astype(np.float64))) * LN2
    return out, lse


def amla_comp_fp32_emulation(Q, K, V, scale, block=64, clamp=-30, with_eps=True, c_reading="appendix", cast="rint",
                            guard=0.0, saturate=True, normalise="b16"):
    """Algorithm 2 with its BF16 scale compensation (Appendix A) in FP32, stated in base 2 with one reference per
    row: mu = rint(m) (the algorithm's -n_i), S32 = 2^(m - mu), S16 = BF16(S32), weights P = 2^(t - ref) with
    ref = m - log2 S16 (so P = 2^(t - m) S16 and the largest weight of a row is S16, BF16-exact), and on every
    block but the first the integer N = 2^23 ((mu_prev - mu) clamped at `clamp`) + 2^23 * 1.5 (c / c_prev - 1) added
    to the accumulator's bit patterns.  Two row sums relative to ref, rescaled by the exact factor
    2^(ref_prev - ref): the FP32 sum of the unrounded weights (gives lse; it equals the algorithm's l_i S16) and
    the sum of the BF16-rounded weights.

    The defaults are the form the kernels take.  The options select what the paper's text fixes differently or
    leaves open:
      c_reading  "appendix": c = S16 / S32 (Appendix A: c_i = r_i / r'_i); "algorithm": the reciprocal, as the
                 assignment in Algorithm 2 reads
      cast       "rint": the shift is an integer by construction and the mantissa term is rounded; "trunc": shift,
                 mantissa term and `guard` are added in FP32 and the product with 2^23 is truncated (Algorithm
                 2's Cast_to_int32 with its 1e-6)
      saturate   True: guarded add (saturating, never past the signed zero); False: the plain wrapping INT32 add
      normalise  "b16": output divided by the sum of the rounded weights; "f32": by the FP32 sum (the
                 algorithm's O / (l_N S16))
      with_eps   False drops the mantissa term (what the compensation buys is then visible)"""
    f32 = np.float32
    G, L = Q.shape[0], K.shape[0]
    O = np.zeros((G, V.shape[1]), dtype=f32)
    l32 = np.zeros(G, dtype=f32)
    l16 = np.zeros(G, dtype=f32)
    m = np.full(G, -np.inf, dtype=f32)
    mu = c_prev = ref = None
    cl2 = f32(scale * math.log2(math.e))
    for lo in range(0, L, block):
        Kb, Vb = K[lo:lo + block], V[lo:lo + block]
        t = (Q @ Kb.T).astype(f32) * cl2
        m = np.maximum(m, t.max(axis=1))
        mu_new = np.rint(m)
        S32 = np.exp2((m - mu_new).astype(f32)).astype(f32)
        S16 = _round_bf16(S32)
        c = (S16 / S32 if c_reading == "appendix" else S32 / S16).astype(f32)
        ref_new = (m - np.log2(S16).astype(f32)).astype(f32)
        P = np.exp2((t - ref_new[:, None]).astype(f32)).astype(f32)
        Pb = _round_bf16(P)
        if mu is not None:
            shift = np.maximum(mu - mu_new, f32(clamp)).astype(f32)
            eps = (f32(1.5) * ((c / c_prev).astype(f32) - f32(1))).astype(f32) if with_eps else np.zeros(G, f32)
            if cast == "rint":
                N = (shift.astype(np.int64) << 23) + np.rint((eps * f32(2.0 ** 23)).astype(f32)).astype(np.int64)
            else:
                N = np.trunc((shift + eps + f32(guard)).astype(f32).astype(np.float64) * 2.0 ** 23).astype(np.int64)
            I = as_int32(O).astype(np.int64)
            if saturate:
                R = np.clip(I + N[:, None], -(1 << 31), (1 << 31) - 1)       # saturating INT32 add
                R = np.maximum(R, np.where(I < 0, -(1 << 31), 0))            # never below the signed zero
            else:
                R = ((I + N[:, None] + (1 << 31)) % (1 << 32)) - (1 << 31)   # wrapping INT32 add
            O = as_fp32(R.astype(np.int32)).copy()
            a = np.exp2((ref - ref_new).astype(f32)).astype(f32)
            l32 = (l32 * a).astype(f32)
            l16 = (l16 * a).astype(f32)
        l32 = (l32 + P.sum(axis=1, dtype=f32)).astype(f32)
        l16 = (l16 + Pb.sum(axis=1, dtype=f32)).astype(f32)
        O = (O + (Pb @ Vb).astype(f32)).astype(f32)
        mu, c_prev, ref = mu_new, c, ref_new
    out = O / (l16 if normalise == "b16" else l32)[:, None]
    lse = (ref.astype(np.float64) + np.log2(l32.astype(np.float64))) * LN2
    return out, lse


def amla_alg2_emulation(Q, K, V, scale, block=512, c_reading="appendix", guard=1e-6):
    """The compensated recurrence with the parameter choices of the paper's own kernel (Algorithm 2, Section 4.2):
    512-key blocks, the truncating cast with its 1e-6, the plain integer add, the output divided by the FP32 row
    sum.  `c_reading` as in amla_comp_fp32_emulation.  Returns the output only."""
    return amla_comp_fp32_emulation(Q, K, V, scale, block=block, c_reading=c_reading, cast="trunc", guard=guard,
                                    saturate=False, normalise="f32")[0]


def flash_fp32_emulation(Q, K, V, scale, block=64):
    """Algorithm 1 ("Base") in FP32 with the exact row max as reference and BF16 P for the PV
    product, the way a mixed-precision kernel runs it (Section 5.1's Base).  Same conventions as
    `amla_fp32_emulation`; returns (out FP32, lse FP64)."""
    f32 = np.float32
    G, L = Q.shape[0], K.shape[0]
    O = np.zeros((G, V.shape[1]), dtype=f32)
    l = np.zeros(G, dtype=f32)
    m = np.full(G, -np.inf, dtype=f32)
    c = f32(scale * math.log2(math.e))
    for lo in range(0, L, block):
        Kb, Vb = K[lo:lo + block], V[lo:lo + block]
        t = (Q @ Kb.T).astype(f32) * c
        m_new = np.maximum(m, t.max(axis=1))
        alpha = np.exp2((m - m_new).astype(f32)).astype(f32)
        P = np.exp2((t - m_new[:, None]).astype(f32)).astype(f32)
        l = (l * alpha + P.sum(axis=1, dtype=f32)).astype(f32)
        O = (O * alpha[:, None] + (_round_bf16(P) @ Vb).astype(f32)).astype(f32)
        m = m_new
    out = O / l[:, None]
    lse = (m.astype(np.float64) + np.log2(l.astype(np.float64))) * LN2
    return out, lse


# --------------------------------------------------------------------------------------
# Section 5.1 error metric
# --------------------------------------------------------------------------------------
def frobenius_error(A, B) -> float:
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    return float(np.linalg.norm(A - B) / (np.linalg.norm(B) + 1e-10))
