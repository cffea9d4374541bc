"""The C-ABI library loads, exports every symbol include/amla.h declares, and its host-side
argument validation returns the documented error codes.  No kernel is launched here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def amla():
    if not os.path.exists(os.path.join(ROOT, "paper_2509_25224_amd", "libamla.so")):
        import __graft_entry__
        __graft_entry__.build()
    from paper_2509_25224_amd import amla as mod
    return mod


def test_every_declared_symbol_is_exported(amla):
    header = open(os.path.join(ROOT, "include", "amla.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(amla_[a-z_]+)\s*\(", header))
    assert declared == set(amla.EXPORTS)
    for name in declared:
        assert getattr(amla.lib, name) is not None


def test_desc_struct_layout_matches_header(amla, tmp_path):
    # 12 int32 fields, then pointer, size_t, pointer, pointer on a 64-bit ABI
    assert ctypes.sizeof(amla.AmlaDesc) == 12 * 4 + 4 * 8
    assert amla.AmlaDesc.workspace.offset == 48
    # and as the C compiler lays the header's struct out
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    fields = [name for name, _ in amla.AmlaDesc._fields_]
    src = tmp_path / "layout.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "amla.h"\nint main(void) {\n'
                   '  printf("%zu\\n", sizeof(amla_desc));\n'
                   + "".join(f'  printf("%zu\\n", offsetof(amla_desc, {f}));\n' for f in fields)
                   + "  return 0;\n}\n")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    got = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert got[0] == ctypes.sizeof(amla.AmlaDesc)
    assert got[1:] == [getattr(amla.AmlaDesc, f).offset for f in fields]


def test_status_strings(amla):
    assert amla.amla_status_string(0) == "ok"
    for st in (-1, -2, -3, -4, -99):
        assert amla.amla_status_string(st)


def _call(amla, desc, q=16, kv=16, tab=16, lens=16, out=16, scale=0.07):
    return amla.lib.amla_decode(q, kv, tab, lens, scale, out, None, ctypes.byref(desc))


def test_argument_validation_error_codes(amla):
    good = amla.make_desc(2, 1, 16, 8, 4)
    assert _call(amla, good, q=None) == amla.AMLA_ERR_NULL_ARG
    assert _call(amla, good, out=None) == amla.AMLA_ERR_NULL_ARG
    assert amla.lib.amla_decode(16, 16, 16, 16, 0.1, 16, None, None) == amla.AMLA_ERR_NULL_ARG
    for field, val in (("d_qk", 512), ("d_v", 576), ("block_size", 128), ("batch", 0), ("s_q", 0),
                       ("num_heads", 0), ("variant", 7), ("num_splits", -1), ("flags", 256), ("reserved", 1)):
        d = amla.make_desc(2, 1, 16, 8, 4)
        setattr(d, field, val)
        assert _call(amla, d) == amla.AMLA_ERR_UNSUPPORTED, field
    assert _call(amla, good, q=24) == amla.AMLA_ERR_UNSUPPORTED          # misaligned pointer
    assert _call(amla, good, scale=float("nan")) == amla.AMLA_ERR_UNSUPPORTED
    assert _call(amla, good, scale=-1.0) == amla.AMLA_ERR_UNSUPPORTED
    comp_lazy = amla.make_desc(2, 1, 16, 8, 4, variant=amla.AMLA_RESCALE_ADD_COMP,
                               flags=amla.AMLA_FLAG_LAZY_RESCALE)
    assert _call(amla, comp_lazy) == amla.AMLA_ERR_UNSUPPORTED           # the compensated reference follows the max
    assert amla.amla_effective_splits(amla.make_desc(2, 1, 16, 8, 4, variant=amla.AMLA_RESCALE_ADD_COMP)) >= 1
    split = amla.make_desc(2, 1, 16, 8, 4, num_splits=2)
    assert _call(amla, split) == amla.AMLA_ERR_WORKSPACE                 # no workspace given
    split.workspace = 4096
    split.workspace_bytes = amla.amla_workspace_bytes(split) - 1
    assert _call(amla, split) == amla.AMLA_ERR_WORKSPACE                 # too small


def test_retired_flag_bits_are_rejected(amla):
    for bit in (4, 64, 256):
        d = amla.make_desc(2, 1, 16, 8, 4, flags=bit)
        assert _call(amla, d) == amla.AMLA_ERR_UNSUPPORTED
        assert amla.amla_effective_splits(d) == 0


def test_iteration_512_exists_for_mul_and_add_of_the_default_family_only(amla):
    it = amla.AMLA_FLAG_ITERATION_512
    for variant in (amla.AMLA_RESCALE_ADD_COMP, amla.AMLA_RESCALE_ADD_LDEXP):
        assert _call(amla, amla.make_desc(2, 1, 16, 8, 4, variant=variant, flags=it)) == amla.AMLA_ERR_UNSUPPORTED
    for variant in (amla.AMLA_RESCALE_MUL, amla.AMLA_RESCALE_ADD):
        t = amla.make_desc(2, 1, 16, 8, 4, variant=variant, flags=it | amla.AMLA_FLAG_TRANSPOSED_ACC)
        assert _call(amla, t) == amla.AMLA_ERR_UNSUPPORTED
        assert amla.amla_effective_splits(amla.make_desc(2, 1, 16, 8, 4, variant=variant, flags=it)) >= 1


def test_balanced_decomposition_is_sized(amla):
    for family in (0, amla.AMLA_FLAG_TRANSPOSED_ACC):
        d = amla.make_desc(32, 2, 128, 5000, 256, flags=amla.AMLA_FLAG_BALANCED | family)
        workers = amla.amla_effective_splits(d)
        assert workers == 128                                    # one workgroup per compute unit (256) over two row tiles
        assert amla.amla_workspace_bytes(d) == (workers + 32 - 1) * 256 * 513 * 4
        assert _call(amla, d) == amla.AMLA_ERR_WORKSPACE         # pieces always need their slots
        c = amla.make_desc(32, 2, 128, 5000, 256, flags=amla.AMLA_FLAG_CAUSAL | family)   # the mask selects the balanced kernels
        assert amla.amla_effective_splits(c) == 128 and amla.amla_workspace_bytes(c) == (128 + 31) * 256 * 513 * 4
    ld = amla.make_desc(32, 2, 128, 5000, 256, variant=amla.AMLA_RESCALE_ADD_LDEXP, flags=amla.AMLA_FLAG_BALANCED)
    assert _call(amla, ld) == amla.AMLA_ERR_UNSUPPORTED


def test_workspace_and_split_queries(amla):
    d = amla.make_desc(128, 2, 128, 8192, 64)
    assert amla.amla_effective_splits(d) == 1 and amla.amla_workspace_bytes(d) == 0
    d = amla.make_desc(64, 1, 128, 4096, 64)
    assert amla.amla_effective_splits(d) == 4
    assert amla.amla_workspace_bytes(d) == 4 * 64 * 128 * 513 * 4
    d = amla.make_desc(8, 4, 128, 8192, 1024)
    assert amla.amla_effective_splits(d) == 8
    d = amla.make_desc(1, 1, 16, 4, 4, num_splits=3)
    assert amla.amla_effective_splits(d) == 3
    bad = amla.make_desc(1, 1, 16, 4, 4, d_qk=128)
    assert amla.amla_effective_splits(bad) == 0 and amla.amla_workspace_bytes(bad) == 0


def test_exponent_add_argument_checks(amla):
    assert amla.lib.amla_exponent_add(None, 16, 4, -1, None) == amla.AMLA_ERR_NULL_ARG
    assert amla.lib.amla_exponent_add(16, 16, 4, 1, None) == amla.AMLA_ERR_UNSUPPORTED
    assert amla.lib.amla_exponent_add(16, 16, 4, -127, None) == amla.AMLA_ERR_UNSUPPORTED
    assert amla.lib.amla_exponent_add(16, 16, 0, -1, None) == amla.AMLA_OK   # nothing to do
