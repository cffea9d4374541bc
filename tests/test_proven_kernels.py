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
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# strict MUL / ADD decode kernels, the split combine kernel, the exponent-add test kernel
PINNED = ("amla_decode_kernelILi0ELb0E", "amla_decode_kernelILi1ELb0E", "amla_combine_kernelE", "amla_exponent_add_kernelE")


def kernel_hashes(tmp):
    sys.path.insert(0, ROOT)
    import __graft_entry__ as entry
    gen = os.path.join(ROOT, "paper_2509_25224_amd", "csrc", "_build")
    for inc in ("amla_decode_gfx950.hsaco.inc", "amla_decode_gfx950_safe.hsaco.inc"):
        if not os.path.exists(os.path.join(gen, inc)):
            os.makedirs(gen, exist_ok=True)
            with open(os.path.join(gen, inc), "w") as f:
                f.write("0,\n")
    flags = [f for f in entry.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    out = os.path.join(tmp, "device.s")
    subprocess.run([HIPCC, *flags, "-I" + gen, "--cuda-device-only", "-S", "-o", out, SRC], check=True,
                   stderr=subprocess.DEVNULL)
    hashes, cur, body = {}, None, []
    for ln in open(out):
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


def test_gpu_proven_kernels_are_instruction_identical(tmp_path):
    if not os.path.exists(HIPCC):
        pytest.skip("no hipcc")
    want = dict(ln.split() for ln in open(GOLD) if ln.strip() and not ln.startswith("#"))
    got = kernel_hashes(str(tmp_path))
    assert set(got) == set(PINNED)
    assert got == want, "a GPU-proven kernel's instruction stream changed: see this file's header"


if __name__ == "__main__" and "--write" in sys.argv:
    import tempfile
    h = kernel_hashes(tempfile.mkdtemp())
    with open(GOLD, "w") as f:
        f.write("# sha256 of the label-normalised gfx950 instruction stream of each compiler-built kernel that has\n"
                "# passed the GPU parity tests (written by tests/test_proven_kernels.py --write)\n")
        for k in PINNED:
            f.write(f"{k} {h[k]}\n")
    print(open(GOLD).read())
