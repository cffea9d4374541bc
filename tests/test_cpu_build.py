"""The decode library's own source -- kernels and host code, unmodified -- compiled for the host against a
stand-in <hip/hip_runtime.h> (tests/cpu_build: one thread per work-item, wave-wide operations as
barriers, direct-to-LDS loads that land only at the wait) and called through the C ABI under
AddressSanitizer on buffers of exactly the documented sizes, against the oracle.  This checks what the
C++ says -- argument checks, split and workspace arithmetic, index arithmetic, masking, softmax state,
the piece walk of the balanced decomposition, synchronisation order -- not what the GPU compiler
makes of it."""
import os
import struct
import subprocess

import numpy as np
import pytest

from oracle import amla_oracle as orc
from paper_2509_25224_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SHIM = os.path.join(ROOT, "tests", "cpu_build")
CLANG = os.path.join(os.environ.get("ROCM_LLVM_BIN", "/opt/rocm/lib/llvm/bin"), "clang++")
MUL, ADD, COMP, LDEXP = 0, 1, 2, 3
NO_SKIP, LAZY, BALANCED, CAUSAL, ITER512, TRANSPOSED = 1, 2, 8, 16, 32, 128
FLAGS = ["-std=c++20", "-O0", "-g", "-fsanitize=address", "-fno-omit-frame-pointer", "-pthread",
         "-Wno-unknown-attributes", "-Wno-ignored-attributes", "-Wno-psabi"]


def build(tmp, extra=()):
    out = str(tmp / "decode_cpu")
    subprocess.run([CLANG, "-x", "c++", *FLAGS, *extra, "-I" + SHIM, "-I" + os.path.join(ROOT, "include"),
                    "-I" + str(tmp), os.path.join(SHIM, "decode_cpu.cpp"), "-o", out], check=True)
    return out


@pytest.fixture(scope="module")
def exe(tmp_path_factory):
    if not os.path.exists(CLANG):
        pytest.skip("no clang++ to build the CPU harness with")
    return build(tmp_path_factory.mktemp("cpu_build"))


def run_cpu(exe, tmp_path, case, variant, flags=0, ns=0, expect_status=0, q_lens=None, static_ws=False):
    inp, outp = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(inp, "wb") as f:
        f.write(struct.pack("<12i", case.batch, case.s_q, case.heads, case.num_blocks, case.max_blocks_per_seq,
                            variant, ns, flags, int(static_ws), int(q_lens is not None), 0, 0))
        f.write(struct.pack("<f", case.softmax_scale))
        for a in (case.q_bits, case.kv_bits, case.block_table, case.seqlens):
            f.write(np.ascontiguousarray(a).tobytes())
        if q_lens is not None:
            f.write(np.ascontiguousarray(np.asarray(q_lens, np.int32)).tobytes())
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0")
    r = subprocess.run([exe, inp, outp], capture_output=True, text=True, env=env, timeout=900)
    assert r.returncode == 0, r.stderr[-3000:]
    raw = np.fromfile(outp, dtype=np.uint8)
    status, splits = (int(x) for x in raw[:8].view(np.int32))
    assert status == expect_status, status
    if status != 0:
        return None, None, splits
    n_rows = case.batch * case.s_q * case.heads
    raw = raw[8:]
    out = raw[:n_rows * 1024].view(np.uint16).astype(np.uint32)
    out = (out << 16).view(np.float32).astype(np.float64).reshape(case.batch, case.s_q, case.heads, 512)
    lse = raw[n_rows * 1024:].view(np.float32).astype(np.float64).reshape(case.batch, case.s_q, case.heads)
    return out, lse, splits


def check(out, lse, case, peaked=False, causal=False, q_lens=None):
    """The GPU tests' bounds: |out error| <= 1e-2 where |exact| < 4, else half a bf16 step + 6e-3 for the
    rounding of the softmax weights; with `peaked` (query scale > 1: few keys carry the weight and the
    outputs reach several units) the second form everywhere, as in the GPU tests' wide-logit cases.
    |lse error| <= 1e-3."""
    want, want_lse = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale,
                                causal=causal, q_lens=q_lens)
    fin = np.isfinite(want_lse)
    assert np.array_equal(lse[~fin], want_lse[~fin])
    half_ulp = 2.0 ** (np.ceil(np.log2(np.maximum(np.abs(want), 2.0 ** -20))) - 9)
    bound = half_ulp + 6e-3 if peaked else np.where(np.abs(want) < 4, 1e-2, half_ulp + 6e-3)
    assert np.all(np.abs(out - want) <= bound), np.abs(out - want).max()
    if fin.any():
        assert np.abs(lse[fin] - want_lse[fin]).max() <= 1e-3


# (variant, flags).  Without a flag the row-rescale kernels run (the default family); AMLA_FLAG_TRANSPOSED_ACC, the
# lazy flag and the ldexp variant select the transposed-accumulator kernels.
KINDS = [pytest.param((MUL, 0), id="mul"), pytest.param((ADD, 0), id="add"), pytest.param((COMP, 0), id="add_comp"),
         pytest.param((MUL, TRANSPOSED), id="mul_t"), pytest.param((ADD, TRANSPOSED), id="add_t"),
         pytest.param((COMP, TRANSPOSED), id="add_comp_t"),
         pytest.param((MUL, LAZY), id="mul_lazy"), pytest.param((ADD, LAZY), id="add_lazy"),
         pytest.param((LDEXP, 0), id="add_ldexp"), pytest.param((LDEXP, LAZY), id="add_ldexp_lazy"),
         pytest.param((MUL, ITER512), id="mul_512"), pytest.param((ADD, ITER512), id="add_512")]


@pytest.mark.parametrize("kind", KINDS)
def test_tiny_config(exe, tmp_path, kind):
    case = wl.make_config(0)
    out, lse, splits = run_cpu(exe, tmp_path, case, kind[0], flags=kind[1])
    assert splits == 1
    check(out, lse, case)


def _ragged(seed, heads=80):
    # lengths 1, 63, empty, 64, 65, and two of a few blocks; heads * s_q = 160 rows: two row tiles, the
    # second with 32 valid rows; spare blocks in the pool and -1 in the unused table entries
    return wl.make_case("edges", seed, batch=7, s_q=2, heads=heads, seqlens=[1, 63, 0, 64, 65, 200, 330], spare_frac=0.25)


@pytest.mark.parametrize("kind,ns", [((MUL, 0), 1), ((ADD, 0), 3), ((COMP, 0), 2), ((MUL, TRANSPOSED), 1), ((ADD, TRANSPOSED), 3),
                                     ((ADD, LAZY), 0), ((LDEXP, 0), 2), ((ADD, ITER512), 3), ((MUL, ITER512), 1)])
def test_ragged_equal_share_splits(exe, tmp_path, kind, ns):
    case = _ragged(51)
    out, lse, splits = run_cpu(exe, tmp_path, case, kind[0], flags=kind[1], ns=ns)
    assert splits == (ns if ns else 1)        # 6 blocks at most per sequence: too short to split by itself
    check(out, lse, case)
    assert np.all(out[2] == 0)


@pytest.mark.parametrize("kind,workers", [((MUL, 0), 3), ((ADD, 0), 8), ((ADD, 0), 41), ((COMP, 0), 1), ((MUL, 0), 5), ((ADD, 0), 0),
                                          ((MUL, TRANSPOSED), 3), ((ADD, TRANSPOSED), 8), ((ADD, LAZY), 41),
                                          ((COMP, TRANSPOSED), 1), ((MUL, LAZY), 5), ((ADD, ITER512), 3),
                                          ((MUL, ITER512), 8)])
def test_ragged_balanced_decomposition(exe, tmp_path, kind, workers):
    """Worker counts below, at and above the number of sequences and (41) above the number of blocks:
    pieces that start mid-sequence, workers that cross several sequences, full pieces written in
    final form, an empty sequence whose zeros come from the combine kernel."""
    case = _ragged(52)
    out, lse, splits = run_cpu(exe, tmp_path, case, kind[0], flags=kind[1] | BALANCED, ns=workers)
    # default: one workgroup per compute unit (256 where no device says otherwise) over the two row tiles,
    # but never more workers than blocks can exist
    assert splits == (workers if workers else min(128, case.batch * case.max_blocks_per_seq))
    check(out, lse, case)
    assert np.all(out[2] == 0)


@pytest.mark.parametrize("kind", [pytest.param((ADD, LAZY), id="add_lazy"), pytest.param((MUL, LAZY), id="mul_lazy"),
                                  pytest.param((COMP, 0), id="add_comp"), pytest.param((COMP, TRANSPOSED), id="add_comp_t"),
                                  pytest.param((MUL, 0), id="mul"), pytest.param((ADD, 0), id="add"),
                                  pytest.param((LDEXP, 0), id="add_ldexp"),
                                  pytest.param((MUL, ITER512), id="mul_512"), pytest.param((ADD, ITER512), id="add_512")])
def test_wide_logits_move_the_reference(exe, tmp_path, kind):
    """Logit spread of tens of base-2 units over 11 blocks: the lazy kernels take the deferred update
    several times, the compensated one rescales with mantissa terms of both signs."""
    case = wl.make_case("wide", 53, batch=1, s_q=1, heads=16, seqlens=[700], q_sigma=8.0)
    out, lse, _ = run_cpu(exe, tmp_path, case, kind[0], flags=kind[1])
    check(out, lse, case, peaked=True)


@pytest.mark.parametrize("family", [0, TRANSPOSED])
def test_no_skip_flag_keeps_the_result(exe, tmp_path, family):
    case = wl.make_case("noskip", 54, batch=1, s_q=1, heads=8, seqlens=[200])
    a = run_cpu(exe, tmp_path, case, ADD, flags=family)
    b = run_cpu(exe, tmp_path, case, ADD, flags=family | NO_SKIP)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    check(b[0], b[1], case)


@pytest.mark.parametrize("kind,workers", [((MUL, 0), 0), ((ADD, 0), 3), ((ADD, 0), 7), ((COMP, 0), 2), ((MUL, 0), 11),
                                          ((MUL, TRANSPOSED), 0), ((ADD, TRANSPOSED), 3), ((ADD, LAZY), 7),
                                          ((COMP, TRANSPOSED), 2), ((MUL, LAZY), 11)])
def test_causal_mask_among_the_query_tokens(exe, tmp_path, kind, workers):
    """s_q = 4 tokens, lengths around block boundaries: tokens with no key at all (kv_len 1), limits that
    end exactly at or fall into the previous block (kv_len 64, 65, 66, 130: whole blocks masked for the
    early tokens, also as the first block of a piece), and 40 heads so that one wave holds rows of two
    tokens.  (Rows that see two or three keys are left out: there the bf16 rounding of two comparable
    weights times the spread of two value rows alone can exceed the bound, mask or no mask.)"""
    case = wl.make_case("causal", 57, batch=7, s_q=4, heads=40, seqlens=[1, 64, 0, 65, 66, 130, 300], spare_frac=0.25)
    out, lse, _ = run_cpu(exe, tmp_path, case, kind[0], flags=kind[1] | CAUSAL, ns=workers)
    check(out, lse, case, causal=True)
    assert np.all(out[0, :3] == 0) and np.all(np.isneginf(lse[0, :3]))
    # and the mask matters: the unmasked result differs
    plain, _ = orc.decode(case.q_bits, case.kv_bits, case.block_table, case.seqlens, case.softmax_scale)
    assert np.abs(out[4, 0] - plain[4, 0]).max() > 0.05


@pytest.mark.parametrize("kind,workers,causal", [((MUL, 0), 0, False), ((ADD, 0), 3, True), ((ADD, 0), 5, False),
                                                 ((COMP, 0), 2, True), ((MUL, 0), 9, True),
                                                 ((MUL, TRANSPOSED), 0, False), ((ADD, TRANSPOSED), 3, True),
                                                 ((ADD, LAZY), 5, False), ((COMP, TRANSPOSED), 2, True), ((MUL, LAZY), 9, True)])
def test_per_sequence_query_counts(exe, tmp_path, kind, workers, causal):
    """q_lens: sequences with all, some, one and none of the s_q = 4 tokens (40 heads: one wave holds rows
    of two tokens, so real and padding rows share a wave), with and without the mask; padding rows come
    back as zeros / -inf whatever the q array holds there."""
    case = wl.make_case("qlens", 58, batch=7, s_q=4, heads=40, seqlens=[1, 64, 0, 65, 200, 130, 300], spare_frac=0.25)
    q_lens = [4, 2, 3, 1, 0, 3, 4]
    flags = kind[1] | (CAUSAL if causal else BALANCED)
    out, lse, _ = run_cpu(exe, tmp_path, case, kind[0], flags=flags, ns=workers, q_lens=q_lens)
    check(out, lse, case, causal=causal, q_lens=q_lens)
    for b, k in enumerate(q_lens):
        assert np.all(out[b, k:] == 0) and np.all(np.isneginf(lse[b, k:]))
    # out-of-range counts are clamped into 0 .. s_q
    wild = [9, -3, 3, 1, 0, 3, 4]
    out2, lse2, _ = run_cpu(exe, tmp_path, case, kind[0], flags=flags, ns=workers, q_lens=wild)
    check(out2, lse2, case, causal=causal, q_lens=[4, 0, 3, 1, 0, 3, 4])


def test_query_counts_select_the_balanced_kernels(exe, tmp_path):
    case = wl.make_config(0)
    out, lse, _ = run_cpu(exe, tmp_path, case, ADD, q_lens=[1])
    check(out, lse, case, q_lens=[1])


def test_auto_split_of_a_long_single_sequence(exe, tmp_path):
    case = wl.make_case("long1", 55, batch=1, s_q=1, heads=128, seqlens=[64 * 16 - 5])
    out, lse, splits = run_cpu(exe, tmp_path, case, ADD)
    assert splits == 4                      # 1 workgroup without splitting; at least 4 blocks per share
    check(out, lse, case)


def test_entry_point_rejects_what_it_documents(exe, tmp_path):
    case = wl.make_config(0)
    run_cpu(exe, tmp_path, case, COMP, flags=LAZY, expect_status=-2)
    run_cpu(exe, tmp_path, case, 7, expect_status=-2)
    run_cpu(exe, tmp_path, case, ADD, flags=4, expect_status=-2)              # flag bits that are not (or no longer) defined
    run_cpu(exe, tmp_path, case, COMP, flags=ITER512, expect_status=-2)       # MUL and ADD of the default family only
    run_cpu(exe, tmp_path, case, ADD, flags=ITER512 | TRANSPOSED, expect_status=-2)
    run_cpu(exe, tmp_path, case, ADD, flags=64, expect_status=-2)
    run_cpu(exe, tmp_path, case, LDEXP, flags=BALANCED, expect_status=-2)     # equal-share kernels only


def test_static_workspace_entry_point(exe, tmp_path):
    """amla_decode_static_workspace against amla_decode, bit for bit: same kernels, the partial results in
    the library's own array instead of the caller's (here an ordinary host array; on the device its address
    comes from hipGetSymbolAddress).  Equal-share splits, the balanced walk, and a shape that needs none."""
    case = _ragged(56)
    for variant, flags, ns in ((ADD, 0, 3), (MUL, BALANCED, 8), (COMP, 0, 1), (ADD, TRANSPOSED, 2)):
        want, want_lse, _ = run_cpu(exe, tmp_path, case, variant, flags=flags, ns=ns)
        got, got_lse, _ = run_cpu(exe, tmp_path, case, variant, flags=flags, ns=ns, static_ws=True)
        assert np.array_equal(got, want) and np.array_equal(got_lse, want_lse, equal_nan=True)
    # what does not fit the array is refused: 20 sequences x 16 splits x 256 rows of 513 floats = 160 MiB > 128 MiB
    big = wl.make_case("big", 57, batch=20, s_q=2, heads=128, seqlens=[64] * 20)
    run_cpu(exe, tmp_path, big, ADD, ns=16, static_ws=True, expect_status=-3)
    run_cpu(exe, tmp_path, big, ADD, ns=12, static_ws=True)                      # 120 MiB: accepted


def test_random_shapes_lengths_and_decompositions(exe, tmp_path):
    """Seeded sweep over small problems: batch, heads, s_q, lengths (with empty sequences and ragged
    last blocks), rescale variant, flags, split factor or worker count."""
    rng = np.random.default_rng(56)
    kinds = [(MUL, 0), (ADD, 0), (COMP, 0), (ADD, NO_SKIP), (MUL, TRANSPOSED), (ADD, TRANSPOSED), (MUL, LAZY), (ADD, LAZY),
             (COMP, TRANSPOSED), (ADD, NO_SKIP | TRANSPOSED)]      # (the 512-key iteration has a sweep of its own below)
    for trial in range(14):
        batch = int(rng.integers(1, 6))
        s_q = int(rng.integers(1, 4))
        heads = int(rng.choice([1, 8, 40, 70]))
        lens = rng.integers(0, 400, batch)
        if rng.random() < 0.5:
            lens[rng.integers(0, batch)] = 0
        variant, flags = kinds[int(rng.integers(0, len(kinds)))]
        balanced = bool(rng.random() < 0.5)
        ns = int(rng.integers(0, 9)) if not balanced else int(rng.integers(0, 12))
        q_sigma = float(rng.choice([1.0, 3.0, 6.0]))
        case = wl.make_case(f"sweep{trial}", 560 + trial, batch=batch, s_q=s_q, heads=heads, seqlens=lens.tolist(),
                            spare_frac=0.3, q_sigma=q_sigma,
                            max_blocks_per_seq=int(lens.max() + 63) // 64 + int(rng.integers(0, 3)) or 1)
        out, lse, _ = run_cpu(exe, tmp_path, case, variant, flags=flags | (BALANCED if balanced else 0), ns=ns)
        check(out, lse, case, peaked=q_sigma > 1.0)


def test_the_harness_notices_a_tile_read_before_it_landed(tmp_path):
    """The stand-in's direct-to-LDS loads land only at the wait.  With the wait planted away the run must
    not pass: the harness is able to see this class of mistake."""
    if not os.path.exists(CLANG):
        pytest.skip("no clang++ to build the CPU harness with")
    bad = build(tmp_path, extra=("-DSHIM_PLANT_NO_WAIT",))
    case = wl.make_config(0)
    inp, outp = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(inp, "wb") as f:
        f.write(struct.pack("<12i", case.batch, case.s_q, case.heads, case.num_blocks, case.max_blocks_per_seq,
                            ADD, 0, 0, 0, 0, 0, 0))
        f.write(struct.pack("<f", case.softmax_scale))
        for a in (case.q_bits, case.kv_bits, case.block_table, case.seqlens):
            f.write(np.ascontiguousarray(a).tobytes())
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0")
    r = subprocess.run([bad, inp, outp], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode != 0 and "loads in flight" in r.stderr


def test_thread_sanitizer_sees_no_race_between_waves(tmp_path):
    """The same program under ThreadSanitizer: the waves of a workgroup share the LDS tile buffers (every
    wave writes its share of a tile, all read all of it), and a buffer refilled or read on the wrong side
    of a barrier is a data race between the threads that stand in for the waves."""
    if not os.path.exists(CLANG):
        pytest.skip("no clang++ to build the CPU harness with")
    exe = str(tmp_path / "decode_tsan")
    subprocess.run([CLANG, "-x", "c++", "-std=c++20", "-O0", "-g", "-fsanitize=thread", "-pthread",
                    "-Wno-unknown-attributes", "-Wno-ignored-attributes", "-Wno-psabi", "-I" + SHIM,
                    "-I" + os.path.join(ROOT, "include"), "-I" + str(tmp_path), os.path.join(SHIM, "decode_cpu.cpp"),
                    "-o", exe], check=True)
    case = wl.make_case("edges", 58, batch=4, s_q=2, heads=80, seqlens=[63, 0, 65, 200], spare_frac=0.25)
    for flags, ns in ((BALANCED, 3), (0, 2), (TRANSPOSED | BALANCED, 3), (TRANSPOSED, 2)):
        out, lse, _ = run_cpu(exe, tmp_path, case, ADD, flags=flags, ns=ns)      # a report makes the exit code non-zero
        check(out, lse, case)


@pytest.mark.parametrize("kind", KINDS)
def test_extreme_inputs(exe, tmp_path, kind):
    """Logits hundreds of base-2 units apart (rescale factors far below 2^-30: the clamp, underflow of the
    multiply, saturation of the guarded add), an all-zero cache (every weight equal, out = 0, lse = ln L,
    zeros that must stay zeros under the exponent add) and a zero query."""
    steep = wl.make_case("steep", 59, batch=1, s_q=1, heads=8, seqlens=[300], q_sigma=30.0)
    out, lse, _ = run_cpu(exe, tmp_path, steep, kind[0], flags=kind[1])
    check(out, lse, steep, peaked=True)
    flat = wl.make_case("flat", 60, batch=2, s_q=1, heads=8, seqlens=[130, 64])
    flat.kv_bits[...] = 0
    out, lse, _ = run_cpu(exe, tmp_path, flat, kind[0], flags=kind[1])
    assert np.all(out == 0)
    assert np.abs(lse - np.log(np.array([130.0, 64.0]))[:, None, None]).max() < 1e-5
    zero_q = wl.make_case("zero_q", 61, batch=1, s_q=1, heads=8, seqlens=[200])
    zero_q.q_bits[...] = 0
    out, lse, _ = run_cpu(exe, tmp_path, zero_q, kind[0], flags=kind[1])
    check(out, lse, zero_q)


def test_the_harness_notices_a_missing_barrier_between_pieces(tmp_path):
    """A copy of the source with the barrier at the start of a piece taken out (a wave may then refill
    an LDS buffer that a slower wave still reads from the previous piece): ThreadSanitizer reports the
    race between the threads that stand in for the waves (whether the race also shows as wrong results
    depends on the timing of a run, so that is not what is asserted).  Planted in a copy, on the CPU."""
    import shutil
    if not os.path.exists(CLANG):
        pytest.skip("no clang++ to build the CPU harness with")
    csrc = tmp_path / "paper_2509_25224_amd" / "csrc"
    csrc.mkdir(parents=True)
    for name in ("amla_decode.hip", "amla_decode_rg.hip", "amla_device.h", "amla_decode_kernels.inc",
                 "amla_decode_equal_share.inc", "amla_decode_piece.inc", "amla_decode_balanced.inc", "amla_plan.h"):
        shutil.copy(os.path.join(ROOT, "paper_2509_25224_amd", "csrc", name), csrc / name)
    piece = (csrc / "amla_decode_rg.hip").read_text()
    barrier = "  // the previous piece's last tile may still be read by a slower wave\n  if (!first_piece) __syncthreads();\n"
    idle = "    if (!first_piece) __syncthreads();\n"          # the same barrier on the path of a wave without rows
    assert barrier in piece and piece.count(idle) == 1
    (csrc / "amla_decode_rg.hip").write_text(piece.replace(barrier, "").replace(idle, ""))
    shim = tmp_path / "tests" / "cpu_build"
    shutil.copytree(os.path.join(SHIM, "hip"), shim / "hip")
    shutil.copy(os.path.join(SHIM, "decode_cpu.cpp"), shim / "decode_cpu.cpp")
    case = wl.make_case("edges", 58, batch=4, s_q=2, heads=80, seqlens=[63, 0, 65, 200], spare_frac=0.25)
    exe = str(tmp_path / "decode_thread")
    subprocess.run([CLANG, "-x", "c++", "-std=c++20", "-O0", "-g", "-fsanitize=thread", "-pthread",
                    "-Wno-unknown-attributes", "-Wno-ignored-attributes", "-Wno-psabi", "-I" + str(shim),
                    "-I" + os.path.join(ROOT, "include"), "-I" + str(tmp_path), str(shim / "decode_cpu.cpp"),
                    "-o", exe], check=True)
    seen = False
    for attempt in range(3):                      # a report makes the exit code non-zero, which run_cpu asserts on
        try:
            run_cpu(exe, tmp_path, case, ADD, flags=BALANCED, ns=2)
        except AssertionError:
            seen = True
            break
    assert seen


@pytest.mark.parametrize("variant", [MUL, ADD, COMP])
def test_row_rescale_kernel(exe, tmp_path, variant):
    """The row-rescale kernels (accumulator laid out query row by register, rescale per moved row): the tiny
    configuration; the ragged case unsplit and in three shares (partial last blocks, an empty sequence and an
    empty share, a second row tile with 32 of 128 rows valid); wide logits that move the reference of many
    rows several times; NaN bit patterns in the cache slots past a sequence's end (the kernel clears them on
    chip); the no-skip flag, which must not change a bit of the ADD variant's result."""
    tiny = wl.make_config(0)
    out, lse, _ = run_cpu(exe, tmp_path, tiny, variant)
    check(out, lse, tiny)
    case = _ragged(71)
    for ns in (1, 3):
        out, lse, splits = run_cpu(exe, tmp_path, case, variant, ns=ns)
        assert splits == ns
        check(out, lse, case)
        assert np.all(out[2] == 0) and np.all(np.isneginf(lse[2]))
    wide = wl.make_case("wide_row", 72, batch=1, s_q=1, heads=40, seqlens=[700], q_sigma=6.0)
    a = run_cpu(exe, tmp_path, wide, variant)
    check(a[0], a[1], wide, peaked=True)
    b = run_cpu(exe, tmp_path, wide, variant, flags=NO_SKIP)
    check(b[0], b[1], wide, peaked=True)
    if variant == ADD:
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    import copy
    dirty = copy.copy(wide)
    dirty.kv_bits = wide.kv_bits.copy()
    phys = int(wide.block_table[0, 700 // 64])
    dirty.kv_bits[phys, 700 % 64:, :] = 0x7FC0          # NaN in every slot past the end of the last block
    c = run_cpu(exe, tmp_path, dirty, variant)
    assert np.array_equal(a[0], c[0]) and np.array_equal(a[1], c[1])


@pytest.mark.parametrize("variant", [MUL, ADD])
def test_iteration_of_512_keys(exe, tmp_path, variant):
    """AMLA_FLAG_ITERATION_512: the reference moves once per eight cache blocks.  Sequences of 24, 9, 8 and 7 blocks
    (an iteration boundary inside, at and past the end), with a ragged last block, whole and in shares that start
    inside an iteration; steep logits (sigma 6: rows leave the kept reference by more than 2^8 and must move it
    at once); the balanced walk and the causal mask."""
    case = wl.make_case("it512", 81, batch=4, s_q=2, heads=40, seqlens=[1500, 570, 512, 448], spare_frac=0.25)
    for flags, ns in ((0, 1), (0, 3), (BALANCED, 5), (CAUSAL, 0)):
        out, lse, _ = run_cpu(exe, tmp_path, case, variant, flags=ITER512 | flags, ns=ns)
        check(out, lse, case, causal=bool(flags & CAUSAL))
    steep = wl.make_case("it512_steep", 84, batch=2, s_q=1, heads=16, seqlens=[1100, 640], q_sigma=6.0)
    for ns in (1, 2):
        out, lse, _ = run_cpu(exe, tmp_path, steep, variant, flags=ITER512, ns=ns)
        check(out, lse, steep, peaked=True)
