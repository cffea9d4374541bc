"""The operand layouts the kernels and the CPU stand-in assume for the two MFMA instructions, against the
lane-mapping constants AMD's ck_tile header ships for them (skipped where the header is not installed).
The 32 x 32 x 16 layout was also measured on the hardware by this build's probes; the 16 x 16 x 32 one of the
eight-wave kernel has only this header and the ISA document behind it so far.

ck_tile's constants: the A/B operand spreads its K index over kABKLane lane groups of kABKPerLane consecutive
elements and its M (N) index over kAMLane (kBNLane) lanes; a C register r of a lane sits in row
(r // kCM1PerLane * kCMLane + lane // kCNLane) * kCM1PerLane + r % kCM1PerLane, column lane % kCNLane."""
import os
import re

import pytest

HEADER = "/opt/rocm/include/ck_tile/ops/gemm/warp/warp_gemm_attribute_mfma_impl.hpp"


def _constants(struct):
    text = open(HEADER).read()
    i = text.index("struct " + struct + "\n")
    body = text[i:text.index("\n};", i)]
    return {k: int(v) for k, v in re.findall(r"static constexpr index_t (k\w+)\s*=\s*(\d+);", body)}


def _c_row(c, r, lane):
    return (r // c["kCM1PerLane"] * c["kCMLane"] + lane // c["kCNLane"]) * c["kCM1PerLane"] + r % c["kCM1PerLane"]


@pytest.mark.skipif(not os.path.exists(HEADER), reason="ck_tile header not installed")
def test_layouts_match_the_ck_tile_header():
    big = _constants("WarpGemmAttributeMfmaImplBf16Bf16F32M32N32K16")
    assert (big["kAMLane"], big["kBNLane"], big["kABKLane"], big["kABKPerLane"]) == (32, 32, 2, 8)
    for lane in range(64):
        for r in range(16):           # measured: row 8 (r // 4) + 4 (lane // 32) + r % 4, column lane % 32
            assert _c_row(big, r, lane) == 8 * (r // 4) + 4 * (lane // 32) + r % 4
    small = _constants("WarpGemmAttributeMfmaImplBf16Bf16F32M16N16K32")
    # A lane l: row l % 16, k = 8 (l // 16) + 0..7; B alike with the column
    assert (small["kAMLane"], small["kBNLane"], small["kABKLane"], small["kABKPerLane"]) == (16, 16, 4, 8)
    assert small["kCNLane"] == 16 and small["kCM0PerLane"] * small["kCM1PerLane"] == 4
    for lane in range(64):
        for r in range(4):            # assumed by the eight-wave kernel: row 4 (lane // 16) + r, column lane % 16
            assert _c_row(small, r, lane) == 4 * (lane // 16) + r
