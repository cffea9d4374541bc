"""Regression guard for the compiler-built kernels that have passed on the GPU: this compiler's register
allocation for the 256-register accumulator does not survive harmless-looking source changes (a shared
lambda cost 50-140 spilled registers, a piece loop crashed the compiler), so the instruction streams of
those kernels are pinned by hash.  A change that is meant to alter them re-runs the GPU tests first and
then rewrites the file: python tests/test_proven_kernels.py --write"""
import hashlib
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLD = os.path.join(ROOT, "tests", "golden", "proven_kernels.sha256")
SRC = os.path.join(ROOT, "paper_2509_25224_amd", "csrc", "amla_decode.hip")
SRC_ROW = os.path.join(ROOT, "paper_2509_25224_amd", "csrc", "amla_decode_rg.hip")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# strict MUL / ADD decode kernels, the split combine kernel, the exponent-add test kernel
PINNED = ("amla_decode_kernelILi0ELb0E", "amla_decode_kernelILi1ELb0E", "amla_combine_kernelILb0EE", "amla_combine_kernelILb1EE",
          "amla_exponent_add_kernelE")


def device_assembly(tmp, src=SRC, name="device.s"):
    """Compiles one source file's device code to gfx950 assembly text; returns the path."""
    sys.path.insert(0, ROOT)
    import __graft_entry__ as entry
    flags = [f for f in entry.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    out = os.path.join(tmp, name)
    subprocess.run([HIPCC, *flags, "--cuda-device-only", "-S", "-o", out, src], check=True,
                   stderr=subprocess.DEVNULL)
    return out


def kernel_hashes(asm_path):
    hashes, cur, body = {}, None, []
    for ln in open(asm_path):
        m = re.match(r"^(_ZN\S+):", ln)
        if m:
            cur, body = m.group(1), []
            continue
        if cur is None:
            continue
        code = re.sub(r";.*", "", ln).strip()
        code = re.sub(r"\.LBB\d+_\d+", "L", code)
        if code:
            body.append(code)
        if code == "s_endpgm":
            for key in PINNED:
                if key in cur:
                    hashes[key] = hashlib.sha256("\n".join(body).encode()).hexdigest()
            cur = None
    return hashes


@pytest.fixture(scope="module")
def asm_path(tmp_path_factory):
    if not os.path.exists(HIPCC):
        pytest.skip("no hipcc")
    return device_assembly(str(tmp_path_factory.mktemp("device_asm")))


def test_gpu_proven_kernels_are_instruction_identical(asm_path):
    want = dict(ln.split() for ln in open(GOLD) if ln.strip() and not ln.startswith("#"))
    got = kernel_hashes(asm_path)
    assert set(got) == set(PINNED)
    assert got == want, "a GPU-proven kernel's instruction stream changed: see this file's header"


def _kernel_bodies(asm_path):
    """name -> list of instruction lines (comments and directives dropped, labels kept)"""
    bodies, cur = {}, None
    for ln in open(asm_path):
        m = re.match(r"^(_ZN\S+):", ln)
        if m:
            cur = m.group(1)
            bodies[cur] = []
            continue
        if cur is None:
            continue
        code = re.sub(r";.*", "", ln).strip()
        if code and not code.startswith("."):
            bodies[cur].append(code)
        elif re.match(r"^\.LBB\d+_\d+:", code or ""):
            bodies[cur].append(code)
        if code == "s_endpgm":
            cur = None
    return bodies


def _steady_loop(body):
    """The instructions from the loop-top barrier to the backward branch that closes the block loop: the
    innermost backward branch region that holds all 136 MFMAs of a block, extended back to its barrier."""
    labels = {ln[:-1]: i for i, ln in enumerate(body) if ln.endswith(":")}
    best = None
    for i, ln in enumerate(body):
        m = re.match(r"s_c?branch\w*\s+(\.LBB\d+_\d+)", ln)
        if m and m.group(1) in labels and labels[m.group(1)] < i:
            a = labels[m.group(1)]
            if sum("v_mfma" in x for x in body[a:i]) >= 136 and (best is None or i - a < best[1] - best[0]):
                best = (a, i)
    assert best is not None
    return body[best[0]:best[1] + 1]


@pytest.fixture(scope="module")
def row_asm_path(tmp_path_factory):
    if not os.path.exists(HIPCC):
        pytest.skip("no hipcc")
    return device_assembly(str(tmp_path_factory.mktemp("device_asm_row")), SRC_ROW, "row.s")


def _check_loads_are_not_serialised(bodies, pattern, expect):
    checked = 0
    for name, body in bodies.items():
        if not re.search(pattern, name):
            continue
        loop = _steady_loop(body)
        issue = [i for i, ln in enumerate(loop) if ln.startswith("s_mov_b32 m0") or ln.startswith("s_add_u32 m0")]
        assert issue, name                                   # the loads are issued inside the loop
        after = loop[issue[0]:]                              # from the first issue point to the closing branch
        assert not [ln for ln in after if ln.startswith("scratch_load")], (name, "reload behind the tile loads")
        assert not [ln for ln in after if ln.startswith("s_waitcnt") and "vmcnt" in ln], (name, "vmcnt wait behind the tile loads")
        checked += 1
    assert checked == expect


def test_tile_loads_are_not_serialised(asm_path, row_asm_path):
    """What the kernels that issue their tile loads from inline assembly are built around, read off the compiled
    loops (one in-order vmcnt for tile loads and scratch reloads; see the comments at AMLA_HIDDEN_LDS_LOAD and
    AMLA_PIECE_LATE_LOADS): inside the block loop no register is reloaded from scratch after the next tile's
    loads were issued, and no vmcnt wait follows them -- only the loop-top wait orders the tile."""
    _check_loads_are_not_serialised(_kernel_bodies(asm_path), r"amla_decode_balanced_kernel", 5)
    _check_loads_are_not_serialised(_kernel_bodies(row_asm_path), r"amla_decode_rg(_balanced)?_kernel", 10)


def test_row_rescale_kernels_keep_the_compiler_out_of_the_accumulator(row_asm_path):
    """The row-rescale kernels address their accumulator, all 256 AccVGPRs, by name from assembly statements:
    compiler-made code must not touch an AccVGPR (the build refuses such a library too), the kernels must be
    allotted all 512 registers, and the loop must be free of scratch traffic."""
    sys.path.insert(0, ROOT)
    import __graft_entry__ as entry
    text = open(row_asm_path).read()
    assert entry.stray_accvgpr_uses(text) == []
    assert text.count(".agpr_count:     256") == 10 and text.count(".vgpr_count:     512") == 10
    for name, body in _kernel_bodies(row_asm_path).items():
        if "amla_decode_rg" in name:
            assert not [ln for ln in _steady_loop(body) if ln.startswith("scratch_")], name


if __name__ == "__main__" and "--write" in sys.argv:
    import tempfile
    h = kernel_hashes(device_assembly(tempfile.mkdtemp()))
    with open(GOLD, "w") as f:
        f.write("# sha256 of the label-normalised gfx950 instruction stream of each compiler-built kernel that has\n"
                "# passed the GPU parity tests (written by tests/test_proven_kernels.py --write)\n")
        for k in PINNED:
            f.write(f"{k} {h[k]}\n")
    print(open(GOLD).read())
