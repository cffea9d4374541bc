"""The generated gfx950 assembly kernels, run on the CPU emulator (tests/gfx950_emu.py) against the
oracle on tiny problems: addressing, pipeline, synchronisation and arithmetic without a GPU."""
import os
import struct
import subprocess
import sys

import numpy as np
import pytest

from oracle import amla_oracle as orc
from paper_2509_25224_amd import workloads as wl
import gfx950_emu as emu
import gfx950_timing as timing

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GEN = os.path.join(ROOT, "paper_2509_25224_amd", "csrc", "gen_decode_asm.py")
LDS_BYTES = 4 * 37 * 1024


@pytest.fixture(scope="module")
def asm_text(tmp_path_factory):
    out = tmp_path_factory.mktemp("asm") / "k.s"
    env = dict(os.environ)
    env.pop("AMLA_ASM_DEBUG", None)
    subprocess.run([sys.executable, GEN, str(out)], check=True, env=env)
    return out.read_text()


def run_case(asm_text, kernel, case, n_splits, flags=0, dma_late=False, smem_first=False, workers=0):
    """`workers` > 0 runs a balanced kernel (name ending in _bal) with that many workers; `n_splits` is
    then ignored."""
    ins, labels = emu.parse_kernel(asm_text, kernel)
    B, T, H = case.batch, case.s_q, case.heads
    rows = T * H
    n_rows = B * rows
    if workers:
        return run_balanced(ins, labels, case, workers, flags, dma_late, smem_first)
    mem = emu.Memory()
    q = mem.add("q", case.q_bits)
    kv = mem.add("kv", case.kv_bits)
    tab = mem.add("table", case.block_table)
    lens = mem.add("seqlens", case.seqlens)
    out = mem.add("out", np.full(n_rows * 512, 0x7F7F, np.uint16), writable=True)
    lse = mem.add("lse", np.full(n_rows, np.nan, np.float32), writable=True)
    po = mem.add("part_o", np.full(max(1, n_splits * n_rows * 512), np.nan, np.float32), writable=True)
    pl = mem.add("part_lse", np.full(max(1, n_splits * n_rows), np.nan, np.float32), writable=True)
    n_streams = B * n_splits
    magic = ((1 << 32) // n_splits + 1) & 0xFFFFFFFF if n_splits > 1 else 0
    scale_log2e = np.float32(case.softmax_scale) * np.float32(1.4426950408889634)
    karg = struct.pack("<8Q", q, kv, tab, lens, out, lse, po, pl) + struct.pack(
        "<f6iIii", float(scale_log2e), B, rows, n_splits, case.max_blocks_per_seq, n_streams, flags, magic,
        case.num_blocks, 0)
    assert len(karg) == 0x68
    ka = mem.add("kernarg", np.frombuffer(karg, dtype=np.uint8))
    n_tiles = (rows + 127) // 128
    gy = (n_streams + 7) // 8
    steps = 0
    for y in range(gy):
        for x in range(8 * n_tiles):
            if y * 8 + (x & 7) >= n_streams and (x, y) != (8 * n_tiles - 1, gy - 1):
                continue                      # padded workgroups exit at once; emulate just one of them
            wg = emu.Workgroup(ins, labels, mem, ka, x, y, LDS_BYTES, dma_late=dma_late, smem_first=smem_first)
            steps += wg.run()
    o = mem.get("out").view(np.uint16).astype(np.uint32)
    o = (o << 16).view(np.float32).astype(np.float64).reshape(B, T, H, 512)
    l = mem.get("lse").view(np.float32).astype(np.float64).reshape(B, T, H)
    if n_splits > 1:
        # merge the partials the way the combine kernel does (exp(lse_s - lse) weights)
        P = mem.get("part_o").view(np.float32).astype(np.float64).reshape(n_splits, n_rows, 512)
        PL = mem.get("part_lse").view(np.float32).astype(np.float64).reshape(n_splits, n_rows)
        mx = PL.max(axis=0)
        with np.errstate(invalid="ignore"):
            w = np.where(np.isneginf(PL), 0.0, np.exp(PL - np.where(np.isneginf(mx), 0.0, mx)))
        tot = w.sum(axis=0)
        with np.errstate(invalid="ignore", divide="ignore"):
            o = np.where(tot[:, None] > 0, (w[:, :, None] * np.nan_to_num(P)).sum(axis=0) / tot[:, None], 0.0)
            l = np.where(tot > 0, mx + np.log(tot), -np.inf)
        o = o.reshape(B, T, H, 512)
        l = l.reshape(B, T, H)
    return o, l, steps


def run_balanced(ins, labels, case, workers, flags, dma_late, smem_first):
    from paper_2509_25224_amd import amla
    B, T, H = case.batch, case.s_q, case.heads
    rows = T * H
    n_rows = B * rows
    slots = workers + B - 1
    mem = emu.Memory()
    q = mem.add("q", case.q_bits)
    kv = mem.add("kv", case.kv_bits)
    tab = mem.add("table", case.block_table)
    lens = mem.add("seqlens", case.seqlens)
    out = mem.add("out", np.full(n_rows * 512, 0x7F7F, np.uint16), writable=True)
    lse = mem.add("lse", np.full(n_rows, np.nan, np.float32), writable=True)
    po = mem.add("part_o", np.full(slots * rows * 512, np.nan, np.float32), writable=True)
    pl = mem.add("part_lse", np.full(slots * rows, np.nan, np.float32), writable=True)
    scale_log2e = np.float32(case.softmax_scale) * np.float32(1.4426950408889634)
    wmagic = ((1 << 32) // workers + 1) & 0xFFFFFFFF
    karg = struct.pack("<8Q", q, kv, tab, lens, out, lse, po, pl) + struct.pack(
        "<f6iIiiiI", float(scale_log2e), B, rows, 1, case.max_blocks_per_seq, workers, flags, 0,
        case.num_blocks, 0, workers, wmagic)
    assert len(karg) == 0x70
    ka = mem.add("kernarg", np.frombuffer(karg, dtype=np.uint8))
    n_tiles = (rows + 127) // 128
    gy = (workers + 7) // 8
    steps = 0
    for y in range(gy):
        for x in range(8 * n_tiles):
            if y * 8 + (x & 7) >= workers and (x, y) != (8 * n_tiles - 1, gy - 1):
                continue
            wg = emu.Workgroup(ins, labels, mem, ka, x, y, LDS_BYTES, dma_late=dma_late, smem_first=smem_first)
            steps += wg.run()
    o = mem.get("out").view(np.uint16).astype(np.uint32)
    o = (o << 16).view(np.float32).astype(np.float64).reshape(B, rows, 512)
    l = mem.get("lse").view(np.float32).astype(np.float64).reshape(B, rows)
    P = mem.get("part_o").view(np.float32).astype(np.float64).reshape(slots, rows, 512)
    PL = mem.get("part_lse").view(np.float32).astype(np.float64).reshape(slots, rows)
    # what the combine kernel does, from the same plan
    lens_c = np.clip(case.seqlens, 0, 64 * case.max_blocks_per_seq)
    pieces, _ = amla.amla_plan_segments(lens_c, workers)
    for b in range(B):
        mine = [p for p in pieces if p[1] == b]
        if not mine:
            o[b], l[b] = 0.0, -np.inf
        elif len(mine) > 1:
            pls = np.stack([PL[p[4]] for p in mine])
            mx = pls.max(axis=0)
            with np.errstate(invalid="ignore"):
                w = np.where(np.isneginf(pls), 0.0, np.exp(pls - np.where(np.isneginf(mx), 0.0, mx)))
            tot = w.sum(axis=0)
            acc = sum(w[i][:, None] * np.nan_to_num(P[p[4]]) for i, p in enumerate(mine))
            with np.errstate(invalid="ignore", divide="ignore"):
                o[b] = np.where(tot[:, None] > 0, acc / tot[:, None], 0.0)
                l[b] = np.where(tot > 0, mx + np.log(tot), -np.inf)
    return o.reshape(B, T, H, 512), l.reshape(B, T, H), steps


def check(o, l, case, bf16_out=True):
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    fin = np.isfinite(want_lse)
    assert np.array_equal(l[~fin], want_lse[~fin])
    eo = np.abs(o - want).max()
    el = np.abs(l[fin] - want_lse[fin]).max() if fin.any() else 0.0
    assert eo <= 1e-2, eo
    assert el <= 1e-3, el
    return eo, el


KERNELS = ["amla_decode_asm_mul", "amla_decode_asm_add", "amla_decode_asm_mul_lazy", "amla_decode_asm_add_lazy",
           "amla_decode_asm_ldexp", "amla_decode_asm_ldexp_lazy"]


def test_generated_assembly_assembles(asm_text, tmp_path):
    """The emulator parses text; the assembler also checks what the text cannot say on this target
    (register-pair alignment, operand kinds, literal counts)."""
    clang = os.path.join(os.environ.get("ROCM_LLVM_BIN", "/opt/rocm/lib/llvm/bin"), "clang")
    if not os.path.exists(clang):
        pytest.skip("no assembler")
    src = tmp_path / "k.s"
    src.write_text(asm_text)
    subprocess.run([clang, "-x", "assembler", "-target", "amdgcn-amd-amdhsa", "-mcpu=gfx950", "-c", str(src), "-o",
                    str(tmp_path / "k.o")], check=True)


def test_hazard_rules_hold(asm_text):
    for k in KERNELS:
        ins, labels = emu.parse_kernel(asm_text, k)
        problems = emu.check_hazards(ins, labels)
        assert not problems, (k, problems[:10])


def test_hazard_checker_sees_the_readfirstlane_mistake():
    """The mistake that faulted the GPU: a VALU write read back by v_readfirstlane in the next slot."""
    text = "k:\n\tv_lshrrev_b32 v252, 6, v251\n\tv_readfirstlane_b32 s36, v252\n\ts_endpgm\n.Lfunc_end_k:\n"
    ins, labels = emu.parse_kernel(text, "k")
    assert emu.check_hazards(ins, labels)


def _problems(body):
    ins, labels = emu.parse_kernel("k:\n" + body + "\ts_endpgm\n.Lfunc_end_k:\n", "k")
    return emu.check_hazards(ins, labels)


def test_hazard_checker_follows_branches_and_counts_nops():
    mfma = "\tv_mfma_f32_32x32x16_bf16 v[144:159], v[200:203], v[0:3], 0\n"
    use = "\tv_add_f32 v176, v144, v160\n"
    assert _problems(mfma + use)                                              # result read at once
    assert _problems(mfma + "\ts_cbranch_scc1 .L_x\n" + "\ts_nop 15\n" * 3 + ".L_x:\n" + use)   # short taken path
    assert not _problems(mfma + "\ts_nop 15\n\ts_nop 3\n" + use)
    assert _problems("\ts_add_u32 m0, s59, 0\n\tglobal_load_lds_dwordx4 v241, s[46:47]\n")
    assert not _problems("\ts_add_u32 m0, s59, 0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 v241, s[46:47]\n")
    assert _problems("\tv_exp_f32 v176, v176\n\tv_add_f32 v253, v176, v177\n")
    assert _problems("\tv_mov_b32 v252, v251\n\ts_nop 0\n\tv_permlane32_swap_b32 v251, v252\n")
    # a dot result: free for the same instruction accumulating into it, three wait states for any other use
    dot = "\tv_dot2c_f32_bf16 v254, s41, v192\n"
    assert not _problems(dot + "\tv_dot2c_f32_bf16 v254, s41, v193\n")
    assert _problems(dot + "\ts_nop 1\n\tv_fma_f32 v240, v240, v250, v254\n")
    assert not _problems(dot + "\ts_nop 2\n\tv_fma_f32 v240, v240, v250, v254\n")
    assert _problems(dot + "\ts_nop 1\n\tv_dot2c_f32_bf16 v253, s41, v254\n")
    assert _problems(dot + "\ts_nop 1\n\tv_mov_b32 v254, 0\n")
    # an SGPR or VCC written by a VALU instruction: two wait states before a VALU instruction reads it
    assert _problems("\tv_cmp_le_i32 vcc, s5, v1\n\tv_cndmask_b32 v2, v2, v3, vcc\n")
    assert _problems("\tv_cmp_le_i32 vcc, s5, v1\n\ts_nop 0\n\tv_cndmask_b32 v2, v2, v3, vcc\n")
    assert not _problems("\tv_cmp_le_i32 vcc, s5, v1\n\ts_nop 1\n\tv_cndmask_b32 v2, v2, v3, vcc\n")
    assert _problems("\tv_add_co_u32 v4, vcc, v4, v6\n\tv_addc_co_u32 v5, vcc, 0, v5, vcc\n")      # the carry of an address
    assert _problems("\tv_readfirstlane_b32 s36, v252\n\tv_add_u32 v1, s36, v1\n")
    assert not _problems("\tv_cmp_gt_i32 vcc, s5, v1\n\ts_and_saveexec_b64 s[56:57], vcc\n")         # scalar readers are interlocked
    acc = "\tv_mfma_f32_32x32x16_bf16 a[0:15], v[200:203], v[0:3], a[0:15]\n"
    assert _problems(acc + "\ts_nop 7\n\tv_accvgpr_read_b32 v5, a3\n")
    assert _problems(acc + "\ts_nop 7\n\tv_accvgpr_write_b32 a3, 0\n")            # overwritten while in flight
    assert not _problems(acc + "\ts_nop 15\n\ts_nop 1\n\tv_accvgpr_write_b32 a3, 0\n")
    assert _problems("\tglobal_store_dwordx4 v[10:11], v[20:23], off\n\tv_mov_b32 v21, 0\n")
    assert not _problems("\tglobal_store_dwordx4 v[10:11], v[20:23], off\n\ts_nop 0\n\tv_mov_b32 v21, 0\n")


def test_emulator_reports_a_missing_wait():
    """A consumer that does not wait for its LDS read is an error, not a silently stale value."""
    text = ("k:\n\tv_mov_b32 v1, 0\n\tds_read_b128 v[200:203], v1 offset:0\n"
            "\tv_add_f32 v2, v200, v200\n\ts_endpgm\n.Lfunc_end_k:\n")
    ins, labels = emu.parse_kernel(text, "k")
    mem = emu.Memory()
    ka = mem.add("kernarg", np.zeros(16, np.uint8))
    wg = emu.Workgroup(ins, labels, mem, ka, 0, 0, 1024)
    wg.lds_write(0, np.zeros(1024, np.uint8))
    with pytest.raises(emu.EmuError):
        wg.run()


@pytest.mark.parametrize("kernel", KERNELS)
def test_tiny_config_on_the_emulator(asm_text, kernel):
    case = wl.make_config(0)                      # 16 heads, kv_len 256: 8 sub-tiles, 16 of 128 rows valid
    o, l, steps = run_case(asm_text, kernel, case, 1)
    check(o, l, case)


@pytest.mark.parametrize("dma_late,smem_first", [(True, False), (False, True), (True, True)])
def test_result_does_not_depend_on_when_loads_land(asm_text, dma_late, smem_first):
    case = wl.make_case("sync", 31, batch=1, s_q=1, heads=8, seqlens=[200], q_sigma=3.0)
    base = run_case(asm_text, "amla_decode_asm_add", case, 1)
    other = run_case(asm_text, "amla_decode_asm_add", case, 1, dma_late=dma_late, smem_first=smem_first)
    assert np.array_equal(base[0], other[0]) and np.array_equal(base[1], other[1])
    check(other[0], other[1], case)


@pytest.mark.parametrize("kernel", ["amla_decode_asm_mul", "amla_decode_asm_add_lazy"])
def test_ragged_lengths_splits_and_empty_sequences(asm_text, kernel):
    # partial sub-tiles (rem < 32), a 33..64 remainder (second half of the block unused), one key,
    # an empty sequence, and split ranges that are empty for short sequences
    case = wl.make_case("ragged", 32, batch=4, s_q=1, heads=4, seqlens=[0, 1, 97, 160], spare_frac=0.5, q_sigma=2.0)
    for ns in (1, 3):
        o, l, _ = run_case(asm_text, kernel, case, ns, dma_late=True)
        check(o, l, case)
        assert np.all(o[0] == 0)


def test_two_row_tiles_and_wide_logits(asm_text):
    # 130 rows -> two workgroups per stream, the second with 2 valid rows; large query scale so
    # that the reference moves and the accumulator rescale path runs in both strict kernels
    case = wl.make_case("tiles", 33, batch=1, s_q=1, heads=130, seqlens=[96], q_sigma=6.0)
    want, _ = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    for kernel in ("amla_decode_asm_mul", "amla_decode_asm_add"):
        o, l, _ = run_case(asm_text, kernel, case, 1)
        half_ulp = 2.0 ** (np.ceil(np.log2(np.maximum(np.abs(want), 1.0))) - 9)
        assert np.all(np.abs(o - want) <= np.where(np.abs(want) < 4, 1e-2, half_ulp + 6e-3))


@pytest.mark.parametrize("kernel", ["amla_decode_asm_mul_lazy", "amla_decode_asm_add_lazy"])
def test_lazy_reference_moves_when_the_max_outruns_it(asm_text, kernel):
    """Logits spread over tens of base-2 units and keys ordered so that the row max keeps growing:
    the lazy kernels must take the deferred update (and the accumulator rescale) several times."""
    case = wl.make_case("lazy", 35, batch=1, s_q=1, heads=8, seqlens=[256], q_sigma=8.0, table="identity")
    # sort the keys of the first head's logits ascending so that later sub-tiles hold larger logits
    q0 = wl.bf16_bits_to_f32(case.q_bits[0, 0, 0]).astype(np.float64)
    kv = wl.bf16_bits_to_f32(case.kv_bits).astype(np.float64).reshape(-1, 576)
    order = np.argsort(kv @ q0)
    case.kv_bits[...] = case.kv_bits.reshape(-1, 576)[order].reshape(case.kv_bits.shape)
    logits = np.sort(kv @ q0) * case.softmax_scale * 1.4426950408889634
    assert logits[-1] - logits[31] > 24                       # the max of sub-tile 0 is outrun by > 3 thresholds
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    o, l, _ = run_case(asm_text, kernel, case, 1)
    half_ulp = 2.0 ** (np.ceil(np.log2(np.maximum(np.abs(want), 1.0))) - 9)
    assert np.all(np.abs(o - want) <= np.where(np.abs(want) < 4, 1e-2, half_ulp + 6e-3))
    assert np.abs(l - want_lse).max() <= 1e-3


def test_no_skip_flag_forces_the_rescale_path(asm_text):
    case = wl.make_case("noskip", 34, batch=1, s_q=1, heads=4, seqlens=[128])
    a = run_case(asm_text, "amla_decode_asm_add", case, 1, flags=0)
    b = run_case(asm_text, "amla_decode_asm_add", case, 1, flags=1)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])     # exponent add of 0 is the identity
    check(b[0], b[1], case)
    c = run_case(asm_text, "amla_decode_asm_mul", case, 1, flags=1)
    check(c[0], c[1], case)


def test_modelled_pass_time_of_the_lazy_kernel(asm_text):
    """Schedule regression guard: in the cycle model a pass (32 keys) of the lazy kernel stays within
    10 % of the 68 back-to-back MFMAs (2176 cycles) it contains."""
    kernel = "amla_decode_asm_add_lazy"
    case = wl.make_case("model", 41, batch=1, s_q=1, heads=128, seqlens=[384])       # 12 passes
    ins, labels = emu.parse_kernel(asm_text, kernel)
    trace = timing.record_trace(lambda: run_case(asm_text, kernel, case, 1))
    per_pass, stall = timing.cycles_per_pass(ins, labels, trace, f".L_{kernel}_loop")
    print(f"modelled cycles per pass: {per_pass:.0f}, stalls {dict(stall)}")
    assert 2176 <= per_pass <= 2176 * 1.10


def test_bad_table_entries_and_lengths_stay_inside_the_buffers(asm_text):
    """A block-table entry outside the pool and a length past the table row are caller mistakes; the
    kernels clamp both, so the result is unspecified but every access stays inside the buffers (the
    emulator's memory raises on any access outside them)."""
    case = wl.make_case("bad", 36, batch=2, s_q=1, heads=4, seqlens=[200, 130], table="identity")
    case.block_table[0, 1] = 1 << 20
    case.block_table[0, 2] = -5
    case.seqlens[1] = 10 ** 6
    for kernel in ("amla_decode_asm_add", "amla_decode_asm_mul_lazy"):
        o, l, _ = run_case(asm_text, kernel, case, 1)
        assert np.all(np.isfinite(o[0]))          # clamped entries point at real blocks


@pytest.mark.parametrize("kernel,workers", [("amla_decode_asm_add_bal", 1), ("amla_decode_asm_mul_bal", 3),
                                            ("amla_decode_asm_add_lazy_bal", 8), ("amla_decode_asm_mul_lazy_bal", 20)])
def test_balanced_walk_on_the_emulator(asm_text, kernel, workers):
    """Worker ranges that start mid-sequence, cross several sequences (with an empty one between) and, with
    20 workers for 12 blocks, are partly empty; pieces written in final form and as partial rows; loads
    that land late, so that a ring refilled too early for the next piece would show."""
    case = wl.make_case("bal", 37, batch=5, s_q=1, heads=4, seqlens=[70, 0, 1, 200, 300], spare_frac=0.5, q_sigma=2.0)
    o, l, _ = run_case(asm_text, kernel, case, 1, dma_late=True, workers=workers)
    check(o, l, case)
    assert np.all(o[1] == 0)


@pytest.mark.parametrize("kernel", ["amla_decode_asm_mul", "amla_decode_asm_add", "amla_decode_asm_add_lazy"])
def test_extreme_inputs_on_the_emulator(asm_text, kernel):
    """Logits hundreds of base-2 units apart (the -30 clamp, underflow of the multiply, saturation of the
    guarded add) and an all-zero cache (out = 0 exactly, lse = ln L)."""
    steep = wl.make_case("steep", 38, batch=1, s_q=1, heads=4, seqlens=[150], q_sigma=30.0)
    want, want_lse = orc.decode(steep.q_bits, steep.kv_bits, steep.block_table, steep.seqlens, steep.softmax_scale)
    o, l, _ = run_case(asm_text, kernel, steep, 1)
    half_ulp = 2.0 ** (np.ceil(np.log2(np.maximum(np.abs(want), 2.0 ** -20))) - 9)
    assert np.all(np.abs(o - want) <= half_ulp + 6e-3)
    assert np.abs(l - want_lse).max() <= 1e-3
    flat = wl.make_case("flat", 39, batch=1, s_q=1, heads=4, seqlens=[100])
    flat.kv_bits[...] = 0
    o, l, _ = run_case(asm_text, kernel, flat, 1)
    assert np.all(o == 0) and np.abs(l - np.log(100.0)).max() < 1e-5


def test_ldexp_kernel_equals_the_integer_add_kernel(asm_text):
    """Same reference, same weights, same products; inside Lemma 3.1's range v_ldexp_f32 and the guarded
    INT32 add are the same operation, so the two kernels' results agree bit for bit.  Wide logits so
    that the rescale path runs, a split so that partial rows are written, a balanced run as well."""
    case = wl.make_case("ldexp", 40, batch=2, s_q=1, heads=8, seqlens=[160, 97], q_sigma=5.0)
    a = run_case(asm_text, "amla_decode_asm_add", case, 2)
    b = run_case(asm_text, "amla_decode_asm_ldexp", case, 2)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    c = run_case(asm_text, "amla_decode_asm_ldexp_bal", case, 1, workers=3)
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    half_ulp = 2.0 ** (np.ceil(np.log2(np.maximum(np.abs(want), 2.0 ** -20))) - 9)
    for o, l, _ in (b, c):
        assert np.all(np.abs(o - want) <= half_ulp + 6e-3)
        assert np.abs(l - want_lse).max() <= 1e-3


def test_random_shapes_on_the_emulator(asm_text):
    """Seeded sweep: batch, heads (one or two row tiles), s_q, lengths with empty sequences and ragged last
    sub-tiles, kernel kind, split factor or worker count, early or late loads."""
    rng = np.random.default_rng(42)
    kinds = ["mul", "add", "ldexp", "mul_lazy", "add_lazy", "ldexp_lazy"]
    for trial in range(6):
        batch = int(rng.integers(1, 5))
        s_q = int(rng.integers(1, 3))
        heads = int(rng.choice([1, 5, 70]))
        lens = rng.integers(0, 230, batch)
        if trial % 2:
            lens[rng.integers(0, batch)] = 0
        kind = kinds[trial % len(kinds)]
        balanced = bool(trial % 2)
        q_sigma = float(rng.choice([1.0, 4.0]))
        case = wl.make_case(f"sweep{trial}", 420 + trial, batch=batch, s_q=s_q, heads=heads, seqlens=lens.tolist(),
                            spare_frac=0.4, q_sigma=q_sigma,
                            max_blocks_per_seq=int(lens.max() + 63) // 64 + int(rng.integers(0, 2)) or 1)
        name = "amla_decode_asm_" + kind + ("_bal" if balanced else "")
        n = int(rng.integers(1, 7))
        o, l, _ = run_case(asm_text, name, case, n, dma_late=bool(rng.integers(0, 2)), workers=n if balanced else 0)
        want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
        fin = np.isfinite(want_lse)
        half_ulp = 2.0 ** (np.ceil(np.log2(np.maximum(np.abs(want), 2.0 ** -20))) - 9)
        assert np.array_equal(l[~fin], want_lse[~fin]), (trial, name)
        assert np.all(np.abs(o - want) <= half_ulp + 6e-3), (trial, name, np.abs(o - want).max())
        if fin.any():
            assert np.abs(l[fin] - want_lse[fin]).max() <= 1e-3, (trial, name)


# ---- the host code's view: arguments recorded from amla_decode in the CPU build, kernel run on the emulator ----
def _host_launch_record(tmp_path, case, variant, flags, num_splits):
    """Builds the library's source for the host (tests/cpu_build), lets amla_decode dispatch a
    hand-scheduled kernel, and returns what it handed to hipModuleLaunchKernel."""
    import test_cpu_build as cpu
    if not os.path.exists(cpu.CLANG):
        pytest.skip("no clang++ to build the CPU harness with")
    exe = cpu.build(tmp_path)
    rec = tmp_path / "launches.bin"
    inp, outp = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(inp, "wb") as f:
        f.write(struct.pack("<12i", case.batch, case.s_q, case.heads, case.num_blocks, case.max_blocks_per_seq,
                            variant, num_splits, flags, 0, 0, 0, 0))
        f.write(struct.pack("<f", case.softmax_scale))
        for a in (case.q_bits, case.kv_bits, case.block_table, case.seqlens):
            f.write(np.ascontiguousarray(a).tobytes())
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", AMLA_ENABLE_BALANCED="1", AMLA_ENABLE_ASM_KERNELS="1",
               AMLA_SHIM_RECORD=str(rec))
    env.pop("LD_PRELOAD", None)
    r = subprocess.run([exe, inp, outp], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    status, splits = (int(x) for x in np.fromfile(outp, dtype=np.int32, count=2))
    assert status == 0, status
    raw = rec.read_bytes()
    n, gx, gy, gz, bx, by, bz, nbytes = struct.unpack_from("<8I", raw, 0)
    name = raw[32:32 + n].decode()
    karg = raw[32 + n:32 + n + nbytes]
    assert len(raw) == 32 + n + nbytes and (gz, bx, by, bz) == (1, 256, 1, 1)
    return name, (gx, gy), karg, splits


@pytest.mark.parametrize("variant,flags,num_splits", [(1, 4, 3), (0, 4 | 2, 0), (3, 4 | 8, 5), (1, 4 | 8 | 2, 0)])
def test_arguments_from_the_host_code_drive_the_kernel(asm_text, tmp_path, variant, flags, num_splits):
    """What amla_decode passes to the hand-scheduled kernels (grid, split factor or worker count, the two
    division constants, pool size), taken from the host code itself, must be what the kernels expect:
    the recorded argument block, with only the eight pointers replaced, runs on the emulator and gives
    the oracle's result.  Flags: 4 = assembly kernels, 2 = lazy, 8 = balanced."""
    from paper_2509_25224_amd import amla
    case = wl.make_case("host", 43, batch=3, s_q=1, heads=6, seqlens=[150, 40, 260], spare_frac=0.3, q_sigma=2.0)
    name, (gx, gy), karg, splits = _host_launch_record(tmp_path, case, variant, flags, num_splits)
    balanced = bool(flags & 8)
    kind = {0: "mul", 1: "add", 3: "ldexp"}[variant]
    assert name == "amla_decode_asm_" + kind + ("_lazy" if flags & 2 else "") + ("_bal" if balanced else "")
    ins, labels = emu.parse_kernel(asm_text, name)
    B, rows = case.batch, case.s_q * case.heads
    n_rows = B * rows
    slots = (splits + B - 1) if balanced else splits * B
    mem = emu.Memory()
    ptrs = [mem.add("q", case.q_bits), mem.add("kv", case.kv_bits), mem.add("table", case.block_table),
            mem.add("seqlens", case.seqlens),
            mem.add("out", np.full(n_rows * 512, 0x7F7F, np.uint16), writable=True),
            mem.add("lse", np.full(n_rows, np.nan, np.float32), writable=True),
            mem.add("part_o", np.full(max(1, slots * rows * 512), np.nan, np.float32), writable=True),
            mem.add("part_lse", np.full(max(1, slots * rows), np.nan, np.float32), writable=True)]
    ka = mem.add("kernarg", np.frombuffer(struct.pack("<8Q", *ptrs) + karg[64:], dtype=np.uint8))
    n_streams = splits if balanced else B * splits
    assert (gx, gy) == (8 * ((rows + 127) // 128), (n_streams + 7) // 8)
    for y in range(gy):
        for x in range(gx):
            if y * 8 + (x & 7) >= n_streams and (x, y) != (gx - 1, gy - 1):
                continue
            emu.Workgroup(ins, labels, mem, ka, x, y, LDS_BYTES, dma_late=True).run()
    o = (mem.get("out").view(np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64).reshape(B, rows, 512)
    l = mem.get("lse").view(np.float32).astype(np.float64).reshape(B, rows)
    P = mem.get("part_o").view(np.float32).astype(np.float64).reshape(-1, rows, 512)
    PL = mem.get("part_lse").view(np.float32).astype(np.float64).reshape(-1, rows)
    if balanced:
        pieces, _ = amla.amla_plan_segments(case.seqlens, splits)
        groups = {b: [p[4] for p in pieces if p[1] == b] for b in range(B)}
    else:
        groups = {b: [s * B + b for s in range(splits)] for b in range(B)} if splits > 1 else {}
    for b, slot_ids in groups.items():
        if len(slot_ids) < 2:
            continue
        pls = np.stack([PL[i] for i in slot_ids])
        mx = pls.max(axis=0)
        w = np.where(np.isneginf(pls), 0.0, np.exp(pls - mx))
        o[b] = sum(w[i][:, None] * np.nan_to_num(P[sid]) for i, sid in enumerate(slot_ids)) / w.sum(axis=0)[:, None]
        l[b] = mx + np.log(w.sum(axis=0))
    check(o.reshape(B, case.s_q, case.heads, 512), l.reshape(B, case.s_q, case.heads), case)


@pytest.mark.parametrize("level", ["1", "waits", "slots"])
def test_the_diagnostic_build_is_the_same_program(tmp_path, level):
    """The padded forms of the kernels (AMLA_ASM_SAFE=1: every wait a full drain and idle slots after
    every instruction, "waits" / "slots": one of the two; the library loads the form built as the
    diagnostic one when AMLA_ASM_SAFE_BUILD=1) assemble, keep the hazard rules and compute the same
    result."""
    out = tmp_path / "safe.s"
    env = dict(os.environ, AMLA_ASM_SAFE=level)
    env.pop("AMLA_ASM_DEBUG", None)
    subprocess.run([sys.executable, GEN, str(out)], check=True, env=env)
    text = out.read_text()
    for kernel in ("amla_decode_asm_add_lazy", "amla_decode_asm_mul_bal"):
        ins, labels = emu.parse_kernel(text, kernel)
        assert emu.check_hazards(ins, labels) == []
    case = wl.make_config(0)
    o, l, _ = run_case(text, "amla_decode_asm_add_lazy", case, 1)
    check(o, l, case)
    clang = os.path.join(os.environ.get("ROCM_LLVM_BIN", "/opt/rocm/lib/llvm/bin"), "clang")
    if os.path.exists(clang):
        subprocess.run([clang, "-x", "assembler", "-target", "amdgcn-amd-amdhsa", "-mcpu=gfx950", "-c", str(out), "-o",
                        str(tmp_path / "safe.o")], check=True)
