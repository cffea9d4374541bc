#!/usr/bin/env python3
"""Generator of the hand-scheduled gfx950 decode kernels (CDNA4 assembly).

Writes one assembly file holding twelve kernels, `amla_decode_asm_{mul,add,ldexp}{,_lazy}{,_bal}`, that
the build assembles into a code object and embeds into libamla.so.  All run the same loop
(Algorithm 1 / Algorithm 2 of the AMLA paper per 32-key sub-tile of a 64-key cache block);
they differ only in how the reference of the exponent is moved and how the accumulator is
rescaled:

  mul        reference = running row max; O *= 2^(m_old - m_new)       (Algorithm 1, Eq. (2))
  add        reference = rint(running row max), an integer power of two; O's bit patterns get
             (n_new - n_old) << 23 added as INT32, guarded against exponent underflow
             (Eq. (4), Lemma 3.1, Algorithm 2's n_i, N and AtomicAdd<INT32> steps)
  ldexp      the add variant with the exponent add done by v_ldexp_f32 (one instruction per register)
  *_bal      balanced decomposition: the workgroup is a worker that walks its share of the batch's
             concatenated block list, one pass through the pipeline per (worker, sequence) piece
  *_lazy     the reference is moved only when the row max exceeds it by more than 2^8; until
             then the softmax weights are allowed to grow up to 2^8 (same relative precision in
             bf16 / FP32), which makes the rescale of the 32 x 512 accumulator a rare event.

Work decomposition: one workgroup = 4 waves = 128 query rows of one (sequence, kv split);
wave w owns rows 32w..32w+31.  Per lane: Q fragment in v0..v143, the 32 x 512 FP32 accumulator
(transposed: lane % 32 is the query row) in a0..a255, everything else in v144..v255.

Pipeline per sub-tile u (32 keys):
  top      wait for sub-tile u+1 (direct-to-LDS loads issued two iterations ago), barrier,
           issue the loads of sub-tile u+3 into the LDS slot that sub-tile u-1 just left
  phase A  S^T(u+1) = K Q^T: 36 MFMAs in two accumulation chains, K operands streamed from LDS;
           interleaved with the online softmax of sub-tile u on the VALU
  rescale  (only if a row of the wave moved its reference) accumulator registers
  phase B  O^T += V^T P^T for sub-tile u: 32 MFMAs, V^T operands through ds_read_b64_tr_b16
LDS: ring of 4 slots of 32 rows x 1168 B (row padded by 16 B so that the 16 rows a b128 read
touches per clock fall into distinct banks), 37 KiB per slot.
"""
from __future__ import annotations

import collections
import os
import sys

ROW = 1168                 # padded LDS row
SLOT = 37 * 1024           # LDS slot: 32 rows * 1168 B = 36.5 KiB, rounded up to whole 1 KiB loads
NSLOT = 4
LDS_BYTES = NSLOT * SLOT   # 151552
LOADS_PER_SUBTILE = 10     # per wave: 9 distinct 1 KiB loads + the shared 37th (issued by every wave)
LAZY_THRESHOLD = 8.0

# ---- VGPR map -------------------------------------------------------------------------------
Q = 0            # 144
SA = 144         # 16  accumulation chain A of S^T(u+1)
SB = 160         # 16  chain B
SC = 176         # 16  scores / weights of sub-tile u
PK = 192         # 8   bf16-packed weights (B operand of phase B)
ST = 200         # 32  operand staging ring, 8 slots of 4
NST = 8
V_M = 232        # running row max (scaled, base 2)
V_REF = 233      # reference subtracted in the exponent
V_L32 = 234      # per-lane partial sum of FP32 weights
V_L16 = 235      # per-lane partial sum of bf16-rounded weights
V_FAC = 236      # mul: alpha, add: n23
V_KOFF = 237
V_VOFF = 238
V_KCUR = 239
V_VCUR = 240
V_LD = 241       # 10 per-lane global offsets of the direct-to-LDS loads
T0, T1, T2, T3, T4 = 251, 252, 253, 254, 255

# ---- SGPR map -------------------------------------------------------------------------------
S_KARG = 0       # 2
S_WGX, S_WGY = 2, 3
S_QP, S_KVP, S_TABP, S_LENP, S_OUTP, S_LSEP, S_POP, S_PLP = 4, 6, 8, 10, 12, 14, 16, 18
S_C, S_BATCH, S_ROWS, S_NS, S_MAXB, S_NSTREAMS, S_FLAGS, S_MAGIC = 20, 21, 22, 23, 24, 25, 26, 27
S_TILE, S_STREAM, S_B, S_SPLIT, S_LEN = 28, 29, 30, 31, 32
S_U, S_ULAST, S_UEND = 33, 34, 35
S_WAVE, S_WAVELDS = 36, 37
S_SLOTV, S_SLOTK, S_SLOTLD = 38, 39, 40
S_ONES = 41
S_TABB = 42      # 2: block-table row of this sequence
S_PHYS = 44
S_GB = 46        # 2: global base of the sub-tile being loaded
S_T0, S_T1, S_T2, S_T3 = 48, 49, 50, 51
S_NEED = 52      # 2
S_FIRST = 54
S_ULD = 55       # sub-tile index the next load targets
S_SAVE = 56      # 2
S_REM = 58
S_M0BASE = 59
S_PHYS2 = 45     # block-table entry fetched one pass ahead
S_ULD2 = 60      # the sub-tile index it belongs to
S_DOIT = 61      # accumulator rescale wanted in this pass
S_GB2 = 62       # 2: global base of the next sub-tile to load
S_UPART = 64     # index of the sub-tile with fewer than 32 keys in range, or -1
S_NBLKM1 = 66    # num_blocks - 1: every block-table entry is clamped into [0, num_blocks - 1]
# balanced decomposition (worker walk over the batch's concatenated block list)
S_WORKERS, S_WMAGIC = 68, 69   # number of workers W, floor(2^32 / W) + 1 (an even-aligned pair: one load)
S_LEFT = 70      # blocks of this worker's range still to process
S_J = 71         # next block of the current sequence
S_J0, S_J1 = 72, 73            # the piece: blocks [j0, j1) of sequence S_B
S_FULL = 74      # the piece covers its whole sequence: write out / lse directly
S_I = 75         # scan index
S_ACC = 76       # scan: blocks before sequence S_I
S_G0 = 77
S_LB = 80        # 16: lengths of one scan chunk (s[80:95])
S_NEXT_FREE = 96

KARG_SIZE = 0x70


class Gen:
    def __init__(self):
        self.lines = []

    def __call__(self, s):
        self.lines.append("\t" + s)

    def label(self, s):
        self.lines.append(s + ":")

    def comment(self, s):
        self.lines.append("\t; " + s)


def vr(base, n=1):
    return f"v{base}" if n == 1 else f"v[{base}:{base + n - 1}]"


def ar(base, n=1):
    return f"a{base}" if n == 1 else f"a[{base}:{base + n - 1}]"


def sr(base, n=1):
    return f"s{base}" if n == 1 else f"s[{base}:{base + n - 1}]"


class LdsQueue:
    """Tracks the order of outstanding LDS reads so that each consumer waits with the exact
    lgkmcnt.  LDS operations return in issue order."""

    def __init__(self):
        self.pending = []
        self.retired = set()

    def issue(self, tag):
        self.retired.discard(tag)
        self.pending.append(tag)
        assert len(self.pending) <= 15

    def wait_for(self, tag):
        """Returns the lgkmcnt value after which `tag` has returned (everything issued before it
        has then returned too).  A tag that an earlier wait already covered needs no wait: the
        value returned is the number of reads outstanding, which the counter cannot exceed."""
        if tag not in self.pending:
            assert tag in self.retired, tag
            return len(self.pending)
        i = self.pending.index(tag)
        n = len(self.pending) - 1 - i
        self.retired.update(self.pending[: i + 1])
        del self.pending[: i + 1]
        return n

    def drain(self):
        self.retired.update(self.pending)
        self.pending.clear()


def issue_cost(ins):
    """Approximate issue cost in cycles of one instruction of the VALU/SALU stream (quarter-rate
    transcendentals, four cycles for everything else, the count of an s_nop)."""
    m = ins.split()[0]
    if m in ("v_exp_f32", "v_log_f32", "v_rcp_f32"):
        return 16
    if m == "s_nop":
        return int(ins.split()[1]) + 1
    return 4


def interleave(g, groups, valu, first_group=0):
    """Emit MFMA groups with the VALU stream spread between them, both in their own order, so that
    the stream's issue cost is spread evenly over the groups from `first_group` on."""
    n = len(groups)
    total = sum(issue_cost(x) for x in valu)
    vi, spent = 0, 0
    for gi, grp in enumerate(groups):
        for ins in grp:
            g(ins)
        if gi < first_group:
            continue
        target = total * (gi - first_group + 1) / (n - first_group)
        while vi < len(valu) and (spent + issue_cost(valu[vi]) / 2 <= target or gi == n - 1):
            g(valu[vi])
            spent += issue_cost(valu[vi])
            vi += 1
    assert vi == len(valu)


def kernel(g: Gen, name: str, rescale: str, lazy: bool, balanced: bool = False):
    L = lambda s: f".L_{name}_{s}"
    g.lines.append(f"\t.globl {name}\n\t.p2align 8\n\t.type {name},@function")
    g.label(name)

    # ------------------------------------------------------------------ prologue: arguments
    g(f"s_load_dwordx16 {sr(S_QP, 16)}, {sr(S_KARG, 2)}, 0x0")
    g(f"s_load_dwordx8 {sr(S_C, 8)}, {sr(S_KARG, 2)}, 0x40")
    g(f"s_load_dword {sr(S_NBLKM1)}, {sr(S_KARG, 2)}, 0x60")
    if balanced:
        g(f"s_load_dwordx2 {sr(S_WORKERS, 2)}, {sr(S_KARG, 2)}, 0x68")
    g(f"v_and_b32 v{T0}, 0x3ff, v0")                            # workitem id x (v0 packs x, y, z)
    g(f"s_and_b32 {sr(S_T0)}, {sr(S_WGX)}, 7")                  # xcd
    g(f"s_lshr_b32 {sr(S_TILE)}, {sr(S_WGX)}, 3")
    g(f"s_lshl_b32 {sr(S_STREAM)}, {sr(S_WGY)}, 3")
    g(f"s_or_b32 {sr(S_STREAM)}, {sr(S_STREAM)}, {sr(S_T0)}")
    g("s_waitcnt lgkmcnt(0)")
    g(f"s_sub_u32 {sr(S_NBLKM1)}, {sr(S_NBLKM1)}, 1")
    if os.environ.get("AMLA_ASM_DEBUG") == "1":
        g("v_mov_b32 v2, 0")
        for i, reg in enumerate((S_WGX, S_WGY, S_STREAM, S_NSTREAMS, S_ROWS, S_NS)):
            g(f"v_mov_b32 v1, {sr(reg)}")
            g(f"v_cvt_f32_i32 v1, v1")
            g(f"global_store_dword v2, v1, {sr(S_LSEP, 2)} offset:{4 * i}")
        g("s_waitcnt vmcnt(0)")
        g("s_endpgm")
    g(f"s_cmp_ge_i32 {sr(S_STREAM)}, {sr(S_NSTREAMS)}")
    g(f"s_cbranch_scc1 {L('end')}")

    def table_row_of_b():
        # block table row: table + b * max_blocks * 4
        g(f"s_mul_i32 {sr(S_T2)}, {sr(S_B)}, {sr(S_MAXB)}")
        g(f"s_mul_hi_u32 {sr(S_T3)}, {sr(S_B)}, {sr(S_MAXB)}")
        g(f"s_lshl_b64 {sr(S_T2, 2)}, {sr(S_T2, 2)}, 2")
        g(f"s_add_u32 {sr(S_TABB)}, {sr(S_TABP)}, {sr(S_T2)}")
        g(f"s_addc_u32 {sr(S_TABB + 1)}, {sr(S_TABP + 1)}, {sr(S_T3)}")

    def wave_id_from_v0():
        g(f"v_lshrrev_b32 v{T1}, 6, v{T0}")
        g("s_nop 3")                                                # VALU write -> v_readfirstlane of the same VGPR needs a wait state
        g(f"v_readfirstlane_b32 {sr(S_WAVE)}, v{T1}")
        g("s_nop 3")
        g(f"s_and_b32 {sr(S_WAVE)}, {sr(S_WAVE)}, 3")               # 4 waves; keeps every derived LDS / global offset in range

    if not balanced:
        # b = stream / n_splits, split = stream % n_splits
        g(f"s_mul_hi_u32 {sr(S_T1)}, {sr(S_STREAM)}, {sr(S_MAGIC)}")
        g(f"s_cmp_eq_u32 {sr(S_NS)}, 1")
        g(f"s_cselect_b32 {sr(S_B)}, {sr(S_STREAM)}, {sr(S_T1)}")
        g(f"s_sub_u32 {sr(S_T1)}, {sr(S_BATCH)}, 1")
        g(f"s_min_u32 {sr(S_B)}, {sr(S_B)}, {sr(S_T1)}")              # b < batch whatever the launch arguments say
        g(f"s_mul_i32 {sr(S_T1)}, {sr(S_B)}, {sr(S_NS)}")
        g(f"s_sub_u32 {sr(S_SPLIT)}, {sr(S_STREAM)}, {sr(S_T1)}")
        g(f"s_lshl_b32 {sr(S_T1)}, {sr(S_B)}, 2")
        g(f"s_load_dword {sr(S_LEN)}, {sr(S_LENP, 2)}, {sr(S_T1)}")
        table_row_of_b()
        # lane decomposition
        wave_id_from_v0()
        g(f"v_and_b32 v{T0}, 63, v{T0}")                            # lane
    else:
        # ---- balanced decomposition: this workgroup is worker S_STREAM of S_WORKERS.  The blocks of all
        # sequences laid end to end are cut into equal worker ranges [w T / W, (w + 1) T / W); the
        # worker walks its range sequence by sequence, one piece (= one turn of the loop below) per
        # sequence it meets.  Divisions by W are mulhi by floor(2^32 / W) + 1, exact while
        # (w + 1) T W < 2^32 (checked by the host).
        wave_id_from_v0()                                           # v0 is overwritten by the first piece's Q loads

        def scan_chunk(per_length):
            """Loads lengths S_I .. S_I + 15 (indices past the end re-read the last one) and hands each,
            as a block count in S_T2 (0 past the end), to per_length(k)."""
            g(f"s_sub_u32 {sr(S_T3)}, {sr(S_BATCH)}, 1")
            for k in range(16):
                g(f"s_add_u32 {sr(S_T1)}, {sr(S_I)}, {k}")
                g(f"s_min_u32 {sr(S_T1)}, {sr(S_T1)}, {sr(S_T3)}")
                g(f"s_lshl_b32 {sr(S_T1)}, {sr(S_T1)}, 2")
                g(f"s_load_dword {sr(S_LB + k)}, {sr(S_LENP, 2)}, {sr(S_T1)}")
            g("s_waitcnt lgkmcnt(0)")
            g(f"s_lshl_b32 {sr(S_T0)}, {sr(S_MAXB)}, 6")                # longest length the table row allows
            for k in range(16):
                g(f"s_max_i32 {sr(S_T2)}, {sr(S_LB + k)}, 0")
                g(f"s_min_i32 {sr(S_T2)}, {sr(S_T2)}, {sr(S_T0)}")
                g(f"s_add_u32 {sr(S_T2)}, {sr(S_T2)}, 63")
                g(f"s_lshr_b32 {sr(S_T2)}, {sr(S_T2)}, 6")              # blocks of sequence S_I + k
                g(f"s_add_u32 {sr(S_T1)}, {sr(S_I)}, {k}")
                g(f"s_cmp_ge_u32 {sr(S_T1)}, {sr(S_BATCH)}")
                g(f"s_cselect_b32 {sr(S_T2)}, 0, {sr(S_T2)}")
                per_length(k)

        # pass 1: T = blocks of the whole batch (in S_ACC)
        g(f"s_mov_b32 {sr(S_I)}, 0")
        g(f"s_mov_b32 {sr(S_ACC)}, 0")
        g.label(L("scan_total"))
        scan_chunk(lambda k: g(f"s_add_u32 {sr(S_ACC)}, {sr(S_ACC)}, {sr(S_T2)}"))
        g(f"s_add_u32 {sr(S_I)}, {sr(S_I)}, 16")
        g(f"s_cmp_lt_u32 {sr(S_I)}, {sr(S_BATCH)}")
        g(f"s_cbranch_scc1 {L('scan_total')}")
        # this worker's range
        g(f"s_mul_i32 {sr(S_T1)}, {sr(S_STREAM)}, {sr(S_ACC)}")         # w T
        g(f"s_add_u32 {sr(S_T2)}, {sr(S_T1)}, {sr(S_ACC)}")              # (w + 1) T
        g(f"s_mul_hi_u32 {sr(S_G0)}, {sr(S_T1)}, {sr(S_WMAGIC)}")
        g(f"s_mul_hi_u32 {sr(S_T2)}, {sr(S_T2)}, {sr(S_WMAGIC)}")
        g(f"s_cmp_eq_u32 {sr(S_WORKERS)}, 1")                            # floor(2^32 / 1) + 1 does not fit 32 bits
        g(f"s_cselect_b32 {sr(S_G0)}, 0, {sr(S_G0)}")
        g(f"s_cselect_b32 {sr(S_T2)}, {sr(S_ACC)}, {sr(S_T2)}")
        g(f"s_sub_u32 {sr(S_LEFT)}, {sr(S_T2)}, {sr(S_G0)}")
        g(f"s_cmp_eq_u32 {sr(S_LEFT)}, 0")
        g(f"s_cbranch_scc1 {L('end')}")
        # pass 2: the sequence that holds block g0: the first i with (blocks before i) + nb_i > g0
        g(f"s_mov_b32 {sr(S_I)}, 0")
        g(f"s_mov_b32 {sr(S_ACC)}, 0")
        g(f"s_mov_b32 {sr(S_B)}, -1")

        def locate(k):
            g(f"s_add_u32 {sr(S_T1)}, {sr(S_ACC)}, {sr(S_T2)}")          # blocks up to and including this sequence
            g(f"s_add_u32 {sr(S_NEED)}, {sr(S_I)}, {k}")                 # candidate sequence
            g(f"s_sub_u32 {sr(S_NEED + 1)}, {sr(S_G0)}, {sr(S_ACC)}")    # and g0's position in it
            g(f"s_cmp_gt_u32 {sr(S_T1)}, {sr(S_G0)}")
            g(f"s_cselect_b32 {sr(S_T3)}, 1, 0")
            g(f"s_cmp_eq_u32 {sr(S_B)}, -1")
            g(f"s_cselect_b32 {sr(S_T3)}, {sr(S_T3)}, 0")                # found here and not found before
            g(f"s_cmp_eq_u32 {sr(S_T3)}, 1")
            g(f"s_cselect_b32 {sr(S_B)}, {sr(S_NEED)}, {sr(S_B)}")
            g(f"s_cselect_b32 {sr(S_J)}, {sr(S_NEED + 1)}, {sr(S_J)}")
            g(f"s_mov_b32 {sr(S_ACC)}, {sr(S_T1)}")
        g(f"s_mov_b32 {sr(S_J)}, 0")
        g.label(L("scan_locate"))
        scan_chunk(locate)
        g(f"s_add_u32 {sr(S_I)}, {sr(S_I)}, 16")
        g(f"s_cmp_lg_u32 {sr(S_B)}, -1")
        g(f"s_cbranch_scc1 {L('located')}")
        g(f"s_cmp_lt_u32 {sr(S_I)}, {sr(S_BATCH)}")
        g(f"s_cbranch_scc1 {L('scan_locate')}")
        g(f"s_branch {L('end')}")                                       # unreachable while g0 < T
        g.label(L("located"))

        # ---- next piece of the walk
        g.label(L("piece_begin"))
        g(f"s_cmp_ge_u32 {sr(S_B)}, {sr(S_BATCH)}")
        g(f"s_cbranch_scc1 {L('end')}")                                 # unreachable while left <= blocks remaining
        g(f"s_lshl_b32 {sr(S_T1)}, {sr(S_B)}, 2")
        g(f"s_load_dword {sr(S_LEN)}, {sr(S_LENP, 2)}, {sr(S_T1)}")
        g("s_waitcnt lgkmcnt(0)")
        g(f"s_max_i32 {sr(S_LEN)}, {sr(S_LEN)}, 0")
        g(f"s_lshl_b32 {sr(S_T0)}, {sr(S_MAXB)}, 6")
        g(f"s_min_i32 {sr(S_LEN)}, {sr(S_LEN)}, {sr(S_T0)}")
        g(f"s_add_u32 {sr(S_T0)}, {sr(S_LEN)}, 63")
        g(f"s_lshr_b32 {sr(S_T0)}, {sr(S_T0)}, 6")                      # nb
        g(f"s_cmp_lt_u32 {sr(S_J)}, {sr(S_T0)}")
        g(f"s_cbranch_scc1 {L('piece_take')}")
        g(f"s_add_u32 {sr(S_B)}, {sr(S_B)}, 1")                         # sequence exhausted or empty: next one
        g(f"s_mov_b32 {sr(S_J)}, 0")
        g(f"s_branch {L('piece_begin')}")
        g.label(L("piece_take"))
        g(f"s_sub_u32 {sr(S_T1)}, {sr(S_T0)}, {sr(S_J)}")               # blocks the sequence still has
        g(f"s_min_u32 {sr(S_T1)}, {sr(S_T1)}, {sr(S_LEFT)}")            # take
        g(f"s_mov_b32 {sr(S_J0)}, {sr(S_J)}")
        g(f"s_add_u32 {sr(S_J1)}, {sr(S_J)}, {sr(S_T1)}")
        g(f"s_sub_u32 {sr(S_LEFT)}, {sr(S_LEFT)}, {sr(S_T1)}")
        g(f"s_mov_b32 {sr(S_J)}, {sr(S_J1)}")
        g(f"s_cmp_eq_u32 {sr(S_J1)}, {sr(S_T0)}")
        g(f"s_cselect_b32 {sr(S_FULL)}, 1, 0")
        g(f"s_cmp_eq_u32 {sr(S_J0)}, 0")
        g(f"s_cselect_b32 {sr(S_FULL)}, {sr(S_FULL)}, 0")
        table_row_of_b()
        # lane decomposition (v0 no longer holds the workitem id)
        g(f"v_mbcnt_lo_u32_b32 v{T0}, -1, 0")
        g(f"v_mbcnt_hi_u32_b32 v{T0}, -1, v{T0}")                    # lane
    g(f"s_lshl_b32 {sr(S_WAVELDS)}, {sr(S_WAVE)}, 10")
    g(f"s_mov_b32 {sr(S_ONES)}, 0x3f803f80")
    g(f"s_mov_b32 {sr(S_FIRST)}, 1")
    # per-lane LDS read offsets
    g(f"v_and_b32 v{T1}, 31, v{T0}")                            # l32
    g(f"v_lshrrev_b32 v{T2}, 5, v{T0}")                         # h
    g(f"v_mul_u32_u24 v{V_KOFF}, {ROW}, v{T1}")
    g(f"v_lshl_add_u32 v{V_KOFF}, v{T2}, 4, v{V_KOFF}")         # l32 * 1168 + h * 16
    g(f"v_lshrrev_b32 v{T3}, 4, v{T0}")                         # g16 = lane >> 4
    g(f"v_and_b32 v{T4}, 15, v{T0}")                            # i16
    g(f"v_lshrrev_b32 v{V_VOFF}, 1, v{T3}")                     # g16 >> 1
    g(f"v_lshlrev_b32 v{V_VOFF}, 2, v{V_VOFF}")                 # 4 * (g16 >> 1)
    g(f"v_lshrrev_b32 v{V_KCUR}, 2, v{T4}")                     # i16 >> 2
    g(f"v_add_u32 v{V_VOFF}, v{V_VOFF}, v{V_KCUR}")
    g(f"v_mul_u32_u24 v{V_VOFF}, {ROW}, v{V_VOFF}")             # row part
    g(f"v_and_b32 v{T3}, 1, v{T3}")                             # g16 & 1
    g(f"v_lshlrev_b32 v{T3}, 5, v{T3}")                         # * 16 columns * 2 B
    g(f"v_and_b32 v{T4}, 3, v{T4}")                             # i16 & 3
    g(f"v_lshl_add_u32 v{T3}, v{T4}, 3, v{T3}")                 # + 4 columns * 2 B each
    g(f"v_add_u32 v{V_VOFF}, v{V_VOFF}, v{T3}")
    # per-lane global offsets of the direct-to-LDS loads: chunk c = 64 i + lane of the padded
    # sub-tile is row c / 73, 16-byte column c % 73 (72 = padding); source offset 16 (c - row)
    for k in range(LOADS_PER_SUBTILE):
        dst = V_LD + k
        if k < 9:
            g(f"s_lshl_b32 {sr(S_T1)}, {sr(S_WAVE)}, 6")
            g(f"s_add_u32 {sr(S_T1)}, {sr(S_T1)}, {256 * k}")    # 64 * (wave + 4 k)
        else:
            g(f"s_mov_b32 {sr(S_T1)}, {36 * 64}")
        g(f"v_add_u32 v{T3}, {sr(S_T1)}, v{T0}")                # c
        g(f"v_mul_u32_u24 v{T4}, 57457, v{T3}")
        g(f"v_lshrrev_b32 v{T4}, 22, v{T4}")                    # row = c / 73
        g(f"v_mul_u32_u24 v{V_KCUR}, 73, v{T4}")
        g(f"v_sub_u32 v{V_KCUR}, v{T3}, v{V_KCUR}")             # c % 73
        g(f"v_sub_u32 v{dst}, v{T3}, v{T4}")
        g(f"v_lshlrev_b32 v{dst}, 4, v{dst}")
        g(f"v_cmp_gt_u32 vcc, 72, v{V_KCUR}")                   # real column
        g(f"v_cmp_gt_u32 {sr(S_NEED, 2)}, 32, v{T4}")           # real row (37th load: lanes 32.. are past the end)
        g(f"s_and_b64 vcc, vcc, {sr(S_NEED, 2)}")
        g(f"v_cndmask_b32 v{dst}, 0, v{dst}, vcc")
        g(f"v_min_u32 v{dst}, {36864 - 16}, v{dst}")             # never past the 32-row half block
    # row of this lane and the Q fragment
    g(f"s_lshl_b32 {sr(S_T1)}, {sr(S_TILE)}, 7")
    g(f"s_lshl_b32 {sr(S_T2)}, {sr(S_WAVE)}, 5")
    g(f"s_add_u32 {sr(S_T1)}, {sr(S_T1)}, {sr(S_T2)}")
    g(f"v_and_b32 v{T1}, 31, v{T0}")
    g(f"v_add_u32 v{V_M}, {sr(S_T1)}, v{T1}")                   # row within the sequence
    g(f"v_cmp_gt_i32 vcc, {sr(S_ROWS)}, v{V_M}")
    g("s_nop 1")                                                 # a VALU-written VCC needs two wait states before a VALU reads it
    g(f"v_cndmask_b32 v{T1}, 0, v{V_M}, vcc")                   # rows past the end read row 0
    g(f"s_mul_i32 {sr(S_T2)}, {sr(S_B)}, {sr(S_ROWS)}")
    g(f"v_add_u32 v{T1}, {sr(S_T2)}, v{T1}")                    # global row
    g(f"v_mov_b32 v{T3}, 1152")
    g(f"v_mad_u64_u32 {vr(V_L32, 2)}, vcc, v{T1}, v{T3}, {sr(S_QP, 2)}")
    g(f"v_lshlrev_b32 v{T2}, 4, v{T2}")                         # h * 16
    g(f"v_add_co_u32 v{V_L32}, vcc, v{V_L32}, v{T2}")
    g("s_nop 1")                                                 # the carry in VCC: two wait states before the VALU that reads it
    g(f"v_addc_co_u32 v{V_L16}, vcc, 0, v{V_L16}, vcc")
    for ks in range(36):
        g(f"global_load_dwordx4 {vr(Q + 4 * ks, 4)}, {vr(V_L32, 2)}, off offset:{32 * ks}")
    # accumulator = 0
    for i in range(256):
        g(f"v_accvgpr_write_b32 a{i}, 0")

    # sub-tile range of this split / piece
    g("s_waitcnt lgkmcnt(0)")
    g(f"s_max_i32 {sr(S_LEN)}, {sr(S_LEN)}, 0")                 # a length outside [0, 64 * max_blocks] must not
    g(f"s_lshl_b32 {sr(S_T0)}, {sr(S_MAXB)}, 6")                # reach past the sequence's block-table row
    g(f"s_min_i32 {sr(S_LEN)}, {sr(S_LEN)}, {sr(S_T0)}")
    g(f"s_add_u32 {sr(S_T0)}, {sr(S_LEN)}, 63")
    g(f"s_lshr_b32 {sr(S_T0)}, {sr(S_T0)}, 6")                  # nb
    g(f"s_add_u32 {sr(S_T1)}, {sr(S_LEN)}, 31")
    g(f"s_lshr_b32 {sr(S_T1)}, {sr(S_T1)}, 5")                  # n32
    if not balanced:
        g(f"s_mul_i32 {sr(S_T2)}, {sr(S_SPLIT)}, {sr(S_T0)}")       # x0 = split * nb
        g(f"s_add_u32 {sr(S_T3)}, {sr(S_T2)}, {sr(S_T0)}")          # x1
        g(f"s_mul_hi_u32 {sr(S_T2)}, {sr(S_T2)}, {sr(S_MAGIC)}")    # j0
        g(f"s_mul_hi_u32 {sr(S_T3)}, {sr(S_T3)}, {sr(S_MAGIC)}")    # j1
        g(f"s_cmp_eq_u32 {sr(S_NS)}, 1")
        g(f"s_cselect_b32 {sr(S_T2)}, 0, {sr(S_T2)}")
        g(f"s_cselect_b32 {sr(S_T3)}, {sr(S_T0)}, {sr(S_T3)}")
    else:
        g(f"s_mov_b32 {sr(S_T2)}, {sr(S_J0)}")
        g(f"s_mov_b32 {sr(S_T3)}, {sr(S_J1)}")
    g(f"s_lshl_b32 {sr(S_U)}, {sr(S_T2)}, 1")                   # u0
    g(f"s_lshl_b32 {sr(S_UEND)}, {sr(S_T3)}, 1")
    g(f"s_min_u32 {sr(S_UEND)}, {sr(S_UEND)}, {sr(S_T1)}")
    g(f"s_sub_u32 {sr(S_ULAST)}, {sr(S_UEND)}, 1")
    # only the last sub-tile of the sequence can be partial: S_REM = kv_len - 32 * (n32 - 1) keys
    g(f"s_sub_u32 {sr(S_T2)}, {sr(S_T1)}, 1")                    # n32 - 1
    g(f"s_lshl_b32 {sr(S_T3)}, {sr(S_T2)}, 5")
    g(f"s_sub_i32 {sr(S_REM)}, {sr(S_LEN)}, {sr(S_T3)}")
    g(f"s_cmp_lt_i32 {sr(S_REM)}, 32")
    g(f"s_cselect_b32 {sr(S_UPART)}, {sr(S_T2)}, -1")
    # state
    g(f"v_mov_b32 v{V_M}, 0xff800000")
    g(f"v_mov_b32 v{V_REF}, 0xff800000")
    g(f"v_mov_b32 v{V_FAC}, 0")

    def finish_state_init():
        g(f"v_mov_b32 v{V_L32}, 0")
        g(f"v_mov_b32 v{V_L16}, 0")

    g(f"s_cmp_ge_u32 {sr(S_U)}, {sr(S_UEND)}")
    g(f"s_cbranch_scc0 {L('nonempty')}")
    g("s_waitcnt vmcnt(0)")
    finish_state_init()
    g(f"s_branch {L('epilogue')}")
    g.label(L("nonempty"))

    # ---- direct-to-LDS load of one sub-tile ---------------------------------------------------
    def tile_base_code(dst=S_GB, phys=S_PHYS, uld=S_ULD):
        """dst = kv + phys * 73728 + (uld & 1) * 36864."""
        return [f"s_max_i32 {sr(phys)}, {sr(phys)}, 0",                 # a table entry outside the pool must not
                f"s_min_i32 {sr(phys)}, {sr(phys)}, {sr(S_NBLKM1)}",    # become a wild address
                f"s_mul_i32 {sr(S_T2)}, {sr(phys)}, 73728",
                f"s_mul_hi_u32 {sr(S_T3)}, {sr(phys)}, 73728",
                f"s_and_b32 {sr(S_T1)}, {sr(uld)}, 1",
                f"s_mul_i32 {sr(S_T1)}, {sr(S_T1)}, 36864",
                f"s_add_u32 {sr(S_T2)}, {sr(S_T2)}, {sr(S_T1)}",
                f"s_addc_u32 {sr(S_T3)}, {sr(S_T3)}, 0",
                f"s_add_u32 {sr(dst)}, {sr(S_KVP)}, {sr(S_T2)}",
                f"s_addc_u32 {sr(dst + 1)}, {sr(S_KVP + 1)}, {sr(S_T3)}"]

    def tile_base_from_phys():
        for ins in tile_base_code():
            g(ins)

    def dma_code(k_lo, k_hi):
        """Loads k_lo .. k_hi-1 of the 10 per wave, into slot S_SLOTLD from S_GB."""
        v = [f"s_add_u32 {sr(S_M0BASE)}, {sr(S_SLOTLD)}, {sr(S_WAVELDS)}"]
        for k in range(k_lo, k_hi):
            if k < 9:
                v.append(f"s_add_u32 m0, {sr(S_M0BASE)}, {4096 * k}")
            else:
                v.append(f"s_add_u32 m0, {sr(S_SLOTLD)}, {36 * 1024}")
            v.append("s_nop 0")
            v.append(f"global_load_lds_dwordx4 v{V_LD + k}, {sr(S_GB, 2)}")
        return v

    def issue_subtile_loads(k_lo=0, k_hi=LOADS_PER_SUBTILE):
        for ins in dma_code(k_lo, k_hi):
            g(ins)

    def fetch_phys_blocking():
        g(f"s_lshr_b32 {sr(S_T1)}, {sr(S_ULD)}, 1")
        g(f"s_lshl_b32 {sr(S_T1)}, {sr(S_T1)}, 2")
        g(f"s_load_dword {sr(S_PHYS)}, {sr(S_TABB, 2)}, {sr(S_T1)}")
        g("s_waitcnt lgkmcnt(0)")

    def advance_slot(reg):
        g(f"s_add_u32 {sr(reg)}, {sr(reg)}, {SLOT}")
        g(f"s_cmp_ge_u32 {sr(reg)}, {LDS_BYTES}")
        g(f"s_cselect_b32 {sr(reg)}, 0, {sr(reg)}")

    # prologue loads: sub-tiles u0 .. u0+3 (clamped to the last one) fill the four slots.  Of the last
    # group only the first half is issued here; the first pass of the loop issues the second half
    # at the place where every later pass completes the group its predecessor started.
    DMA_SPLIT = 5
    g(f"s_mov_b32 {sr(S_SLOTLD)}, 0")
    for n in range(NSLOT):
        g(f"s_add_u32 {sr(S_ULD)}, {sr(S_U)}, {n}")
        g(f"s_min_u32 {sr(S_ULD)}, {sr(S_ULD)}, {sr(S_ULAST)}")
        fetch_phys_blocking()
        tile_base_from_phys()
        if n < NSLOT - 1:
            issue_subtile_loads()
            advance_slot(S_SLOTLD)
        else:
            issue_subtile_loads(0, DMA_SPLIT)                    # S_GB and S_SLOTLD stay set for the second half
    g(f"s_mov_b32 {sr(S_SLOTV)}, 0")
    g(f"s_mov_b32 {sr(S_SLOTK)}, 0")
    # block-table entry of sub-tile min(u0+4, last), whose loads the first pass starts after its barrier
    g(f"s_add_u32 {sr(S_ULD2)}, {sr(S_U)}, {NSLOT}")
    g(f"s_min_u32 {sr(S_ULD2)}, {sr(S_ULD2)}, {sr(S_ULAST)}")
    g(f"s_lshr_b32 {sr(S_T1)}, {sr(S_ULD2)}, 1")
    g(f"s_lshl_b32 {sr(S_T1)}, {sr(S_T1)}, 2")
    g(f"s_load_dword {sr(S_PHYS2)}, {sr(S_TABB, 2)}, {sr(S_T1)}")
    g("s_waitcnt lgkmcnt(0)")
    finish_state_init()

    # ---- operand ring -------------------------------------------------------------------------
    # One pass consumes 68 MFMA operands from LDS: K_0..K_35 (one b128 read each) for S^T(u+1), then
    # V_0..V_31 (two transposing b64 reads each) for O^T(u).  Operand number n of a pass of parity p
    # lives in ring slot (n + 4 p) % 8, and the fetch of operand n + 8 is issued right after the MFMA
    # that consumed operand n, into the slot that MFMA just freed.  68 % 8 = 4, so the slot phase
    # alternates between passes; the loop body is unrolled twice (p = 0, 1).
    def ring(n, p):
        return ST + 4 * ((n + 4 * p) % NST)

    def k_fetch(ks, p):
        return [f"ds_read_b128 {vr(ring(ks, p), 4)}, v{V_KCUR} offset:{32 * ks}"]

    order = [(st, dt) for st in range(2) for dt in range(16)]

    def v_fetch(idx, p):
        st, dt = order[idx]
        slot = ring(36 + idx, p)
        base = st * 16 * ROW + dt * 64
        return [f"ds_read_b64_tr_b16 {vr(slot, 2)}, v{V_VCUR} offset:{base}",
                f"ds_read_b64_tr_b16 {vr(slot + 2, 2)}, v{V_VCUR} offset:{base + 8 * ROW}"]

    def qk_mfma(ks, p):
        dst = SA if ks % 2 == 0 else SB
        src_c = "0" if ks < 2 else vr(dst, 16)
        return (f"v_mfma_f32_32x32x16_bf16 {vr(dst, 16)}, {vr(ring(ks, p), 4)}, {vr(Q + 4 * ks, 4)}, {src_c}")

    def pv_mfma(idx, p):
        st, dt = order[idx]
        return (f"v_mfma_f32_32x32x16_bf16 {ar(16 * dt, 16)}, {vr(ring(36 + idx, p), 4)}, "
                f"{vr(PK + 4 * st, 4)}, {ar(16 * dt, 16)}")

    def set_k_base():
        g(f"v_add_u32 v{V_KCUR}, {sr(S_SLOTK)}, v{V_KOFF}")

    def prologue_qk():
        """S^T of the first sub-tile, not overlapped with anything: its own K fetches, parity 0."""
        q = LdsQueue()
        set_k_base()
        for ks in range(NST):
            for ins in k_fetch(ks, 0):
                g(ins)
            q.issue(ks)
        for ks in range(36):
            g(f"s_waitcnt lgkmcnt({q.wait_for(ks)})")
            g(qk_mfma(ks, 0))
            if ks + NST < 36:
                for ins in k_fetch(ks + NST, 0):
                    g(ins)
                q.issue(ks + NST)

    # ---- softmax of the scores in SC (VALU stream) -------------------------------------------
    def softmax_stream():
        v = []
        sc = [SC + r for r in range(16)]
        v.append(f"v_max3_f32 v{T0}, v{sc[0]}, v{sc[1]}, v{sc[2]}")
        for i in range(3, 15, 2):
            v.append(f"v_max3_f32 v{T0}, v{T0}, v{sc[i]}, v{sc[i + 1]}")
        v.append(f"v_max_f32 v{T0}, v{T0}, v{sc[15]}")
        v.append(f"v_mov_b32 v{T1}, v{T0}")
        v.append("s_nop 3")
        v.append(f"v_permlane32_swap_b32 v{T0}, v{T1}")
        v.append("s_nop 3")
        v.append(f"v_max_f32 v{T0}, v{T0}, v{T1}")
        v.append(f"v_mul_f32 v{T0}, {sr(S_C)}, v{T0}")
        v.append(f"v_max_f32 v{T0}, v{V_M}, v{T0}")                      # m_new
        v.append(f"v_mov_b32 v{V_M}, v{T0}")
        # candidate reference
        if rescale in ("add", "ldexp"):
            v.append(f"v_rndne_f32 v{T1}, v{T0}")
        else:
            v.append(f"v_mov_b32 v{T1}, v{T0}")
        if lazy:
            v.append(f"v_add_f32 v{T4}, {LAZY_THRESHOLD}, v{V_REF}")
            v.append(f"v_cmp_gt_f32 vcc, v{T0}, v{T4}")
            v.append("s_nop 1")                                  # VCC from a VALU: two wait states before a VALU reads it
            v.append(f"v_cndmask_b32 v{T1}, v{V_REF}, v{T1}, vcc")      # keep the old reference unless exceeded
        # factor on the old state, and whether any row of the wave needs the accumulator rescaled
        if rescale == "mul":
            v.append(f"v_sub_f32 v{T4}, v{V_REF}, v{T1}")
            v.append(f"v_exp_f32 v{V_FAC}, v{T4}")
            v.append(f"v_cmp_neq_f32 {sr(S_NEED, 2)}, v{V_REF}, v{T1}")
        else:
            v.append(f"v_sub_f32 v{T4}, v{V_REF}, v{T1}")                # <= 0, integer valued (or -inf)
            v.append(f"v_max_f32 v{T4}, 0xc1f00000, v{T4}")             # clamp at -30 (Algorithm 2's max(n_i - n_{i-1}, -30))
            if rescale == "add":
                v.append(f"v_cvt_i32_f32 v{T4}, v{T4}")
                v.append(f"v_lshlrev_b32 v{V_FAC}, 23, v{T4}")              # n * 2^23 for the integer add
            else:
                v.append(f"v_cvt_i32_f32 v{V_FAC}, v{T4}")                  # n itself for v_ldexp_f32
            v.append(f"v_cmp_ne_u32 {sr(S_NEED, 2)}, 0, v{V_FAC}")
        v.append(f"v_mov_b32 v{V_REF}, v{T1}")
        # weights 2^(s * c - ref), their FP32 sum, the bf16 pack and the sum of the rounded weights.
        # The quarter-rate exponentials are spaced out between the cheaper instructions that
        # consume earlier results (each at least two instructions after its producer).
        work = collections.deque()           # cheap consumers waiting to be placed
        for r in range(16):
            v.append(f"v_fma_f32 v{sc[r]}, v{sc[r]}, {sr(S_C)}, -v{T1}")
            if work:
                v.append(work.popleft())
            v.append(f"v_exp_f32 v{sc[r]}, v{sc[r]}")
            if work:
                v.append(work.popleft())
            if r == 1:
                work.append(f"v_add_f32 v{T2}, v{sc[0]}, v{sc[1]}")
            elif r > 1:
                work.append(f"v_add_f32 v{T2}, v{T2}, v{sc[r]}")
            if r % 2 == 1:
                i = r // 2
                work.append(f"v_cvt_pk_bf16_f32 v{PK + i}, v{sc[2 * i]}, v{sc[2 * i + 1]}")
                if i == 0:
                    work.append(f"v_mov_b32 v{T3}, 0")
                work.append(f"v_dot2c_f32_bf16 v{T3}, {sr(S_ONES)}, v{PK + i}")      # T3 += lo + hi of the packed pair
        v.append("s_nop 0")
        v.extend(work)
        if rescale == "mul":
            v.append(f"v_fma_f32 v{V_L32}, v{V_L32}, v{V_FAC}, v{T2}")
            v.append("s_nop 1")                                  # a dot result needs three wait states before another
            v.append(f"v_fma_f32 v{V_L16}, v{V_L16}, v{V_FAC}, v{T3}")    # instruction may read it
        elif rescale == "ldexp":
            for reg, add in ((V_L32, T2), (V_L16, T3)):
                v.append(f"v_ldexp_f32 v{reg}, v{reg}, v{V_FAC}")
                v.append(f"v_add_f32 v{reg}, v{reg}, v{add}")
        else:
            for reg, add in ((V_L32, T2), (V_L16, T3)):
                v.append(f"v_and_b32 v{T4}, 0x80000000, v{reg}")
                v.append(f"v_add_i32 v{reg}, v{reg}, v{V_FAC} clamp")
                v.append(f"v_max_i32 v{reg}, v{reg}, v{T4}")
                v.append(f"v_add_f32 v{reg}, v{reg}, v{add}")
        return v

    def form_scores_stream():
        """SC = SA + SB once the chains have drained."""
        return [f"v_add_f32 v{SC + r}, v{SA + r}, v{SB + r}" for r in range(16)]

    def mask_partial():
        """Keys >= S_REM of the sub-tile whose scores are in SC get -inf."""
        # lane's key for register r: 4 h + 8 (r >> 2) + (r & 3); h = lane >> 5
        g(f"v_mbcnt_lo_u32_b32 v{T0}, -1, 0")
        g(f"v_mbcnt_hi_u32_b32 v{T0}, -1, v{T0}")                 # lane id
        g(f"v_lshrrev_b32 v{T0}, 5, v{T0}")
        g(f"v_lshlrev_b32 v{T0}, 2, v{T0}")                       # 4 h
        g(f"v_mov_b32 v{T1}, 0xff800000")
        for r in range(16):
            const = 8 * (r >> 2) + (r & 3)
            g(f"s_sub_i32 {sr(S_T1)}, {sr(S_REM)}, {const}")      # key >= rem  <=>  4 h >= rem - const
            g(f"v_cmp_le_i32 vcc, {sr(S_T1)}, v{T0}")
            g("s_nop 1")                                          # VCC from a VALU: two wait states before a VALU reads it
            g(f"v_cndmask_b32 v{SC + r}, v{SC + r}, v{T1}, vcc")

    # ---- prologue: scores of sub-tile u0, then the first K fetches of sub-tile u0+1 --------------
    g(f"s_waitcnt vmcnt({2 * LOADS_PER_SUBTILE + DMA_SPLIT})")  # Q fragment and sub-tile u0 have landed
    g("s_barrier")
    prologue_qk()
    g("s_nop 15")
    g("s_nop 15")
    for ins in form_scores_stream():
        g(ins)
    g(f"s_cmp_lg_u32 {sr(S_U)}, {sr(S_UPART)}")
    g(f"s_cbranch_scc1 {L('pro_full')}")
    mask_partial()
    g.label(L("pro_full"))
    advance_slot(S_SLOTK)                                       # slot of sub-tile u0 + 1
    g(f"s_waitcnt vmcnt({LOADS_PER_SUBTILE + DMA_SPLIT})")      # sub-tile u0 + 1 has landed
    g("s_barrier")
    set_k_base()
    lq = LdsQueue()                                             # carried through both passes of the loop body
    for ks in range(NST):
        for ins in k_fetch(ks, 0):
            g(ins)
        lq.issue(("K", 0, ks))

    def rescale_path(tag):
        """Accumulator rescale (rare path), eight registers at a time through SC, which is free
        between the end of the softmax and the score adds of the second half of the pass."""
        g(f"s_cmp_eq_u32 {sr(S_DOIT)}, 0")
        g(f"s_cbranch_scc1 {L('no_rescale' + tag)}")
        for base in range(0, 256, 8):
            for r in range(8):
                g(f"v_accvgpr_read_b32 v{SC + r}, a{base + r}")
            if rescale == "mul":
                for r in range(8):
                    g(f"v_mul_f32 v{SC + r}, v{SC + r}, v{V_FAC}")
            elif rescale == "ldexp":
                for r in range(8):
                    g(f"v_ldexp_f32 v{SC + r}, v{SC + r}, v{V_FAC}")
            else:
                for r in range(8):
                    g(f"v_and_b32 v{SC + 8 + r}, 0x80000000, v{SC + r}")
                for r in range(8):
                    g(f"v_add_i32 v{SC + r}, v{SC + r}, v{V_FAC} clamp")
                for r in range(8):
                    g(f"v_max_i32 v{SC + r}, v{SC + r}, v{SC + 8 + r}")
            for r in range(8):
                g(f"v_accvgpr_write_b32 a{base + r}, v{SC + r}")
        g("s_nop 7")
        g.label(L("no_rescale" + tag))

    def rescale_flag_code():
        """S_DOIT = (some row of the wave moved its reference, or NO_SKIP) and not the first pass."""
        return [f"s_cmp_lg_u64 {sr(S_NEED, 2)}, 0",
                f"s_cselect_b32 {sr(S_DOIT)}, 1, 0",
                f"s_bitcmp1_b32 {sr(S_FLAGS)}, 0",                # AMLA_FLAG_NO_SKIP
                f"s_cselect_b32 {sr(S_T1)}, 1, 0",
                f"s_or_b32 {sr(S_DOIT)}, {sr(S_DOIT)}, {sr(S_T1)}",
                f"s_andn2_b32 {sr(S_DOIT)}, {sr(S_DOIT)}, {sr(S_FIRST)}",
                f"s_mov_b32 {sr(S_FIRST)}, 0"]

    N_K, N_V = 36, 32
    N_USE = N_K + N_V
    BARRIER_AFTER = N_K + 26          # the barrier of the pass follows the MFMA of operand V_26

    def one_pass(p):
        """Pass for sub-tile u with ring parity p.  On entry: scores of u in SC; sub-tiles u and u+1
        resident, u+2 and u+3 landed or in flight; K_0..K_7 of sub-tile u+1 in flight;
        S_SLOTV = slot(u), V_KCUR = K base of slot(u+1)."""
        tag = f"_p{p}"
        g(f"v_add_u32 v{V_VCUR}, {sr(S_SLOTV)}, v{V_VOFF}")
        ready = []                     # fetches whose ring slot is free, in order: (tag, instructions)

        def fetch_of(n):
            """Fetch of operand n of this pass, or of operand n - 68 of the next pass."""
            if n < N_K:
                return ("K", p, n), k_fetch(n, p), False
            if n < N_USE:
                return ("V", p, n - N_K), v_fetch(n - N_K, p), False
            return ("K", 1 - p, n - N_USE), k_fetch(n - N_USE, 1 - p), True      # next sub-tile: only after the barrier

        def consume(n, barrier_passed):
            grp = []
            kind = ("K", p, n) if n < N_K else (("V", p, n - N_K), 1)      # a V operand is complete with its second read
            grp.append(f"s_waitcnt lgkmcnt({min(lq.wait_for(kind), 15)})")
            grp.append(qk_mfma(n, p) if n < N_K else pv_mfma(n - N_K, p))
            ready.append(fetch_of(n + NST))
            while ready:
                t, instrs, after_barrier = ready[0]
                if after_barrier and not barrier_passed:
                    break
                if len(lq.pending) + len(instrs) > 15:
                    break
                ready.pop(0)
                grp.extend(instrs)
                for k in range(len(instrs)):
                    lq.issue(t if len(instrs) == 1 else (t, k))
            return grp

        # -- first half: QK of sub-tile u+1 under the softmax of sub-tile u; from K_28 on the freed
        #    ring slots already take V^T operands of the second half, which moves a quarter of the
        #    transposing reads into the half whose LDS load is light
        groups = []
        for n in range(N_K):
            grp = []
            grp.extend(consume(n, False))
            groups.append(grp)
        # VALU/SALU stream of the first half: the second half of the direct-to-LDS loads that the
        # previous pass started, the softmax, the rescale decision
        # The block-table entry fetched during the previous pass (its arrival was covered by that
        # pass's lgkmcnt(0)) gives the base of the sub-tile whose loads start after this pass's
        # barrier; then the entry for the pass after is fetched.  SMEM shares lgkmcnt with LDS and may
        # return out of order; counting only the LDS reads in the waits stays correct (an outstanding
        # SMEM op can only make a wait stricter), and the wait before the barrier is lgkmcnt(0).
        table_code = tile_base_code(S_GB2, S_PHYS2, S_ULD2) + [
            f"s_add_u32 {sr(S_ULD2)}, {sr(S_U)}, {NSLOT + 1}",
            f"s_min_u32 {sr(S_ULD2)}, {sr(S_ULD2)}, {sr(S_ULAST)}",
            f"s_lshr_b32 {sr(S_T1)}, {sr(S_ULD2)}, 1",
            f"s_lshl_b32 {sr(S_T1)}, {sr(S_T1)}, 2",
            f"s_load_dword {sr(S_PHYS2)}, {sr(S_TABB, 2)}, {sr(S_T1)}"]
        interleave(g, groups, dma_code(DMA_SPLIT, LOADS_PER_SUBTILE) + table_code + softmax_stream()
                   + rescale_flag_code())

        rescale_path(tag)

        # -- second half, body: PV MFMAs 0..24 with the remaining V^T fetches
        groups = [consume(n, False) for n in range(N_K, BARRIER_AFTER + 1)]
        # the score adds read the results of the last QK MFMAs: they start four groups in, more than
        # 30 issue slots after the last QK MFMA
        interleave(g, groups, form_scores_stream(), first_group=4)
        assert all(not (t[0] == "V") for t, _, _ in ready), "every V fetch must be out before the barrier"

        # -- barrier of the pass.  lgkmcnt(0): every V^T read of slot(u) by this wave has returned (and
        #    the block-table entry); vmcnt: of the two load groups in flight (u+2, u+3) the older has
        #    landed.  After the barrier that holds for all waves: slot(u) may be refilled and
        #    sub-tile u+2 may be read.
        g(f"s_waitcnt vmcnt({LOADS_PER_SUBTILE}) lgkmcnt(0)")
        lq.drain()
        g("s_barrier")
        advance_slot(S_SLOTK)                                   # slot(u+2)
        set_k_base()
        g(f"s_mov_b32 {sr(S_SLOTLD)}, {sr(S_SLOTV)}")
        g(f"s_mov_b64 {sr(S_GB, 2)}, {sr(S_GB2, 2)}")
        # -- second half, tail: the last PV MFMAs run after the barrier, each freeing the ring slot
        #    that the next K fetch of sub-tile u+2 refills; the direct-to-LDS loads of sub-tile
        #    min(u+4, last) into slot(u) are issued in between
        first = []
        while ready and len(lq.pending) + len(ready[0][1]) <= 15:
            t, instrs, _ = ready.pop(0)
            first.extend(instrs)
            lq.issue(t)
        for ins in first:
            g(ins)
        groups = [consume(n, True) for n in range(BARRIER_AFTER + 1, N_USE)]
        advance = [f"s_add_u32 {sr(S_U)}, {sr(S_U)}, 1",
                   f"s_add_u32 {sr(S_SLOTV)}, {sr(S_SLOTV)}, {SLOT}",
                   f"s_cmp_ge_u32 {sr(S_SLOTV)}, {LDS_BYTES}",
                   f"s_cselect_b32 {sr(S_SLOTV)}, 0, {sr(S_SLOTV)}"]
        interleave(g, groups, dma_code(0, DMA_SPLIT) + advance)
        assert not ready

        # -- next pass, the end, or first the mask of a partial last sub-tile (its scores are in SC now)
        g(f"s_cmp_ge_u32 {sr(S_U)}, {sr(S_UEND)}")
        g(f"s_cbranch_scc1 {L('epilogue')}")
        g(f"s_cmp_lg_u32 {sr(S_U)}, {sr(S_UPART)}")
        g(f"s_cbranch_scc1 {L('full' + tag)}")
        mask_partial()
        g.label(L("full" + tag))

    # ------------------------------------------------------------------------------ main loop
    g.label(L("loop"))
    one_pass(0)
    one_pass(1)
    assert [t for t in lq.pending] == [("K", 0, ks) for ks in range(NST)], lq.pending
    g(f"s_branch {L('loop')}")

    # --------------------------------------------------------------------------------- epilogue
    DONE = L('piece_done') if balanced else L('end')      # where a wave goes when it has nothing (more) to store
    g.label(L("epilogue"))
    g("s_waitcnt vmcnt(0) lgkmcnt(0)")
    if os.environ.get("AMLA_ASM_DEBUG") == "2":
        g(f"v_mov_b32 v{T0}, 0")
        for i, reg in enumerate((S_U, S_UEND, S_LEN, S_SPLIT, S_B, S_TILE, S_WAVE, S_ULAST)):
            g(f"v_mov_b32 v{T1}, {sr(reg)}")
            g(f"v_cvt_f32_i32 v{T1}, v{T1}")
            g(f"global_store_dword v{T0}, v{T1}, {sr(S_LSEP, 2)} offset:{4 * i}")
        for i, reg in enumerate((V_M, V_REF, V_L32, V_L16, V_FAC, SC, SC + 1, PK)):
            g(f"global_store_dword v{T0}, v{reg}, {sr(S_LSEP, 2)} offset:{32 + 4 * i}")
        g("s_waitcnt vmcnt(0)")
        g("s_endpgm")
    g("s_nop 15")
    g("s_nop 15")
    # totals over the two lane halves
    for reg in (V_L32, V_L16):
        g(f"v_mov_b32 v{T1}, v{reg}")
        g("s_nop 3")
        g(f"v_permlane32_swap_b32 v{reg}, v{T1}")
        g("s_nop 3")
        g(f"v_add_f32 v{reg}, v{reg}, v{T1}")
    g(f"v_rcp_f32 v{T2}, v{V_L16}")
    g(f"v_cmp_lt_f32 vcc, 0, v{V_L16}")
    g("s_nop 1")                                                 # trans result above; VCC: two wait states before a VALU reads it
    g(f"v_cndmask_b32 v{T2}, 0, v{T2}, vcc")                     # 1 / l (0 for an empty range)
    g(f"v_log_f32 v{T3}, v{V_L32}")
    g("s_nop 0")
    g(f"v_add_f32 v{T3}, v{T3}, v{V_REF}")
    g(f"v_mul_f32 v{T3}, 0x3f317218, v{T3}")                    # * ln 2
    g(f"v_cmp_lt_f32 vcc, 0, v{V_L32}")
    g(f"v_mov_b32 v{T4}, 0xff800000")
    g("s_nop 0")                                                 # second wait state between the VCC write and its VALU read
    g(f"v_cndmask_b32 v{T3}, v{T4}, v{T3}, vcc")                 # lse (-inf for an empty range)
    # row index and store mask
    g(f"v_mbcnt_lo_u32_b32 v{T0}, -1, 0")
    g(f"v_mbcnt_hi_u32_b32 v{T0}, -1, v{T0}")                    # lane
    g(f"v_lshrrev_b32 v{V_KOFF}, 5, v{T0}")                      # h
    g(f"v_and_b32 v{T0}, 31, v{T0}")
    g(f"s_lshl_b32 {sr(S_T1)}, {sr(S_TILE)}, 7")
    g(f"s_lshl_b32 {sr(S_T2)}, {sr(S_WAVE)}, 5")
    g(f"s_add_u32 {sr(S_T1)}, {sr(S_T1)}, {sr(S_T2)}")
    g(f"v_add_u32 v{T0}, {sr(S_T1)}, v{T0}")                     # row
    g(f"v_cmp_gt_i32 vcc, {sr(S_ROWS)}, v{T0}")
    g(f"s_and_saveexec_b64 {sr(S_SAVE, 2)}, vcc")
    g(f"s_cbranch_execz {DONE}")
    g(f"s_mul_i32 {sr(S_T2)}, {sr(S_B)}, {sr(S_ROWS)}")
    g(f"v_add_u32 v{T0}, {sr(S_T2)}, v{T0}")                     # global row  b * rows + row
    g(f"s_cmp_eq_u32 {sr(S_FULL if balanced else S_NS)}, 1")     # whole sequence in one piece / no split: final form
    g(f"s_cbranch_scc0 {L('store_partial')}")

    # direct: bf16 out + lse
    g(f"v_mov_b32 v{T4}, 1024")
    g(f"v_mad_u64_u32 {vr(V_L32, 2)}, vcc, v{T0}, v{T4}, {sr(S_OUTP, 2)}")
    g(f"v_lshlrev_b32 v{T4}, 3, v{V_KOFF}")                      # h * 8 B
    g(f"v_add_co_u32 v{V_L32}, vcc, v{V_L32}, v{T4}")
    g("s_nop 1")                                                 # the carry in VCC: two wait states before the VALU that reads it
    g(f"v_addc_co_u32 v{V_L16}, vcc, 0, v{V_L16}, vcc")
    if os.environ.get("AMLA_ASM_DEBUG") == "3":
        g(f"v_mov_b32 v{V_VOFF}, 0")
        g(f"v_mov_b32 v{V_KCUR}, exec_lo")
        g(f"v_cvt_f32_u32 v{V_KCUR}, v{V_KCUR}")
        g(f"global_store_dword v{V_VOFF}, v{V_KCUR}, {sr(S_LSEP, 2)} offset:0")
        g(f"v_cvt_f32_u32 v{V_KCUR}, v{V_L32}")
        g(f"global_store_dword v{V_VOFF}, v{V_KCUR}, {sr(S_LSEP, 2)} offset:4")
        g(f"v_cvt_f32_u32 v{V_KCUR}, v{V_L16}")
        g(f"global_store_dword v{V_VOFF}, v{V_KCUR}, {sr(S_LSEP, 2)} offset:8")
        g(f"v_mov_b32 v{V_KCUR}, {sr(S_OUTP)}")
        g(f"v_cvt_f32_u32 v{V_KCUR}, v{V_KCUR}")
        g(f"global_store_dword v{V_VOFF}, v{V_KCUR}, {sr(S_LSEP, 2)} offset:12")
        g(f"v_mov_b32 v{V_KCUR}, {sr(S_OUTP + 1)}")
        g(f"v_cvt_f32_u32 v{V_KCUR}, v{V_KCUR}")
        g(f"global_store_dword v{V_VOFF}, v{V_KCUR}, {sr(S_LSEP, 2)} offset:16")
        g(f"global_store_dword v{V_VOFF}, v{T2}, {sr(S_LSEP, 2)} offset:20")
        g(f"global_store_dword v{V_VOFF}, v{T3}, {sr(S_LSEP, 2)} offset:24")
        g(f"v_accvgpr_read_b32 v{V_KCUR}, a0")
        g(f"global_store_dword v{V_VOFF}, v{V_KCUR}, {sr(S_LSEP, 2)} offset:28")
        g("s_waitcnt vmcnt(0)")
        g("s_endpgm")
    for dt in range(16):
        for rg in range(4):
            t = ST + 8 * (rg % 4)
            for e in range(4):
                g(f"v_accvgpr_read_b32 v{t + e}, a{16 * dt + 4 * rg + e}")
            for e in range(4):
                g(f"v_mul_f32 v{t + e}, v{t + e}, v{T2}")
            g(f"v_cvt_pk_bf16_f32 v{t + 4}, v{t}, v{t + 1}")
            g(f"v_cvt_pk_bf16_f32 v{t + 5}, v{t + 2}, v{t + 3}")
            g(f"global_store_dwordx2 {vr(V_L32, 2)}, {vr(t + 4, 2)}, off offset:{64 * dt + 16 * rg}")
    g(f"s_cmp_eq_u64 {sr(S_LSEP, 2)}, 0")
    g(f"s_cbranch_scc1 {DONE}")
    g(f"v_cmp_eq_u32 vcc, 0, v{V_KOFF}")                         # h == 0 writes the row's lse
    g(f"s_and_b64 exec, exec, vcc")
    g(f"s_cbranch_execz {DONE}")
    g(f"v_mov_b32 v{T4}, 4")
    g(f"v_mad_u64_u32 {vr(V_L32, 2)}, vcc, v{T0}, v{T4}, {sr(S_LSEP, 2)}")
    g(f"global_store_dword {vr(V_L32, 2)}, v{T3}, off")
    g(f"s_branch {DONE}")

    # split: f32 partial out + partial lse at [(split * batch * rows) + global row]
    g.label(L("store_partial"))
    if not balanced:
        g(f"s_mul_i32 {sr(S_T1)}, {sr(S_BATCH)}, {sr(S_ROWS)}")
        g(f"s_mul_i32 {sr(S_T1)}, {sr(S_T1)}, {sr(S_SPLIT)}")
    else:
        # slot worker + sequence: partial row (w + b) * rows + row = w * rows + global row
        g(f"s_mul_i32 {sr(S_T1)}, {sr(S_STREAM)}, {sr(S_ROWS)}")
    g(f"v_add_u32 v{T0}, {sr(S_T1)}, v{T0}")
    g(f"v_mov_b32 v{T4}, 2048")
    g(f"v_mad_u64_u32 {vr(V_L32, 2)}, vcc, v{T0}, v{T4}, {sr(S_POP, 2)}")
    g(f"v_lshlrev_b32 v{T4}, 4, v{V_KOFF}")                      # h * 16 B
    g(f"v_add_co_u32 v{V_L32}, vcc, v{V_L32}, v{T4}")
    g("s_nop 1")                                                 # the carry in VCC: two wait states before the VALU that reads it
    g(f"v_addc_co_u32 v{V_L16}, vcc, 0, v{V_L16}, vcc")
    for dt in range(16):
        for rg in range(4):
            t = ST + 4 * ((4 * dt + rg) % 8)
            for e in range(4):
                g(f"v_accvgpr_read_b32 v{t + e}, a{16 * dt + 4 * rg + e}")
            for e in range(4):
                g(f"v_mul_f32 v{t + e}, v{t + e}, v{T2}")
            g(f"global_store_dwordx4 {vr(V_L32, 2)}, {vr(t, 4)}, off offset:{128 * dt + 32 * rg}")
    g(f"v_cmp_eq_u32 vcc, 0, v{V_KOFF}")
    g(f"s_and_b64 exec, exec, vcc")
    g(f"s_cbranch_execz {DONE}")
    g(f"v_mov_b32 v{T4}, 4")
    g(f"v_mad_u64_u32 {vr(V_L32, 2)}, vcc, v{T0}, v{T4}, {sr(S_PLP, 2)}")
    g(f"global_store_dword {vr(V_L32, 2)}, v{T3}, off")

    if balanced:
        # the piece is done; the next one refills the LDS ring, which a slower wave may still be reading
        g.label(L("piece_done"))
        g("s_mov_b64 exec, -1")
        g("s_waitcnt vmcnt(0) lgkmcnt(0)")
        g("s_barrier")
        g(f"s_cmp_lg_u32 {sr(S_LEFT)}, 0")
        g(f"s_cbranch_scc1 {L('piece_begin')}")
    g.label(L("end"))
    g("s_endpgm")
    g.lines.append(f".Lfunc_end_{name}:\n\t.size {name}, .Lfunc_end_{name}-{name}")

    # kernel descriptor
    g.lines.append(f"""
	.rodata
	.p2align 6
	.amdhsa_kernel {name}
		.amdhsa_group_segment_fixed_size {LDS_BYTES}
		.amdhsa_private_segment_fixed_size 0
		.amdhsa_kernarg_size {KARG_SIZE}
		.amdhsa_user_sgpr_count 2
		.amdhsa_user_sgpr_kernarg_segment_ptr 1
		.amdhsa_system_sgpr_workgroup_id_x 1
		.amdhsa_system_sgpr_workgroup_id_y 1
		.amdhsa_system_sgpr_workgroup_id_z 0
		.amdhsa_system_vgpr_workitem_id 0
		.amdhsa_next_free_vgpr 512
		.amdhsa_next_free_sgpr {S_NEXT_FREE}
		.amdhsa_accum_offset 256
		.amdhsa_reserve_vcc 1
		.amdhsa_float_round_mode_32 0
		.amdhsa_float_round_mode_16_64 0
		.amdhsa_float_denorm_mode_32 3
		.amdhsa_float_denorm_mode_16_64 3
		.amdhsa_dx10_clamp 1
		.amdhsa_ieee_mode 1
	.end_amdhsa_kernel
	.text
""")


def metadata(names):
    out = ["\t.amdgpu_metadata", "---", "amdhsa.kernels:"]
    for name in names:
        out.append(f"""  - .agpr_count:     256
    .args:
      - .offset:         0
        .size:           {KARG_SIZE}
        .value_kind:     by_value
    .group_segment_fixed_size: {LDS_BYTES}
    .kernarg_segment_align: 8
    .kernarg_segment_size: {KARG_SIZE}
    .max_flat_workgroup_size: 256
    .name:           {name}
    .private_segment_fixed_size: 0
    .sgpr_count:     {S_NEXT_FREE + 6}
    .sgpr_spill_count: 0
    .symbol:         {name}.kd
    .uniform_work_group_size: 1
    .uses_dynamic_stack: false
    .vgpr_count:     512
    .vgpr_spill_count: 0
    .wavefront_size: 64""")
    out += ["amdhsa.target:   amdgcn-amd-amdhsa--gfx950", "amdhsa.version:", "  - 1", "  - 2", "...", "",
            "\t.end_amdgpu_metadata"]
    return "\n".join(out)


KERNELS = [(f"amla_decode_asm_{kind}{'_lazy' if lazy else ''}{'_bal' if bal else ''}", kind, lazy, bal)
           for bal in (False, True) for lazy in (False, True) for kind in ("mul", "add", "ldexp")]


def main():
    out_path = sys.argv[1]
    g = Gen()
    g.lines.append('\t.amdgcn_target "amdgcn-amd-amdhsa--gfx950"')
    g.lines.append("\t.text")
    for name, rescale, lazy, balanced in KERNELS:
        kernel(g, name, rescale, lazy, balanced)
    level = os.environ.get("AMLA_ASM_SAFE", "")
    if level in ("1", "waits", "slots"):
        # Diagnostic build: every wait is a full drain ("waits"), every instruction is followed by idle
        # issue slots ("slots"), or both ("1"), so that a wrong result that disappears here points at a
        # counted wait or at a wait-state rule respectively.
        safe = []
        for ln in g.lines:
            t = ln.strip()
            if t.startswith("s_waitcnt") and level != "slots":
                safe.append("\ts_waitcnt vmcnt(0) lgkmcnt(0)")
                continue
            safe.append(ln)
            if level == "waits":
                continue
            if t.startswith("v_mfma"):
                safe.append("\ts_nop 15")
                safe.append("\ts_nop 3")
            elif t.startswith(("v_", "ds_", "global_", "s_add_u32 m0")):
                safe.append("\ts_nop 4")
        g.lines = safe
    text = "\n".join(g.lines) + "\n" + metadata([k[0] for k in KERNELS]) + "\n"
    with open(out_path, "w") as f:
        f.write(text)


if __name__ == "__main__":
    main()
