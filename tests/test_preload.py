"""The library's Preload Pipeline rotation (amla_preload_rotation, host only) against the oracle's
timeline definition.  Several rotations can be admissible, so the comparison is: the library's choice is
one of the oracle's admissible rotations, equal to it where that is unique; its other outputs follow
from the choice."""
import os
import random
import sys

import pytest

sys.path.insert(0, os.path.join(os.path.dirname(__file__), "..", "oracle"))
import preload_oracle as po  # noqa: E402

amla = pytest.importorskip("paper_2509_25224_amd.amla")


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 8, 13])
def test_choice_is_admissible(n):
    rng = random.Random(n)
    unique = 0
    for trial in range(2000):
        cube = [rng.randint(0, 60) for _ in range(n)]
        vec = [rng.randint(0, 60) for _ in range(n)]
        if trial % 4 == 0:                                   # tight: the vector stages use the whole Cycle
            vec = [0] * n
            for _ in range(sum(cube)):
                vec[rng.randrange(n)] += 1
        if sum(vec) > sum(cube):
            with pytest.raises(amla.AmlaError):
                amla.amla_preload_rotation(cube, vec)
            continue
        first, external, count = amla.amla_preload_rotation(cube, vec)
        want = po.admissible_rotations(cube, vec)
        assert first in want, (cube, vec, first, want)
        if len(want) == 1:
            unique += 1
            assert first == want[0]
        assert external == po.cube_order(n, first)[-1]
        assert count == po.preload_count(n, n - 1) == n
    assert n == 1 or unique > 20


def test_the_chain_of_this_library():
    """n = 2, V2 = 0 (Section 4.1, 'Preload Pipeline for AMLA'): always the Cycle that ends with C1."""
    rng = random.Random(3)
    for _ in range(300):
        c1, c2 = rng.randint(1, 9000), rng.randint(0, 9000)
        v1 = rng.randint(0, c1 + c2)
        assert amla.amla_preload_rotation([c1, c2], [v1, 0]) == (2, 1, 2)


def test_rejections():
    import ctypes
    with pytest.raises(amla.AmlaError):
        amla.amla_preload_rotation([], [])
    with pytest.raises(amla.AmlaError):
        amla.amla_preload_rotation([5, -1], [1, 1])
    with pytest.raises(amla.AmlaError):
        amla.amla_preload_rotation([1 << 62, 1], [0, 0])
    out = ctypes.c_int32(0)
    assert amla.lib.amla_preload_rotation(None, None, 2, ctypes.byref(out), ctypes.byref(out),
                                          ctypes.byref(out)) == amla.AMLA_ERR_NULL_ARG


def test_the_block_loop_is_the_cycle_the_rule_picks_for_its_measured_stages():
    """The decode kernels' block loop works a 64-key block as two 32-key sub-blocks in the order
    C1(0), C1(1) | V1(0), C2(0) | V1(1), C2(1): seen from one sub-block, its vector stage runs beside the matrix
    stage that follows its own C1, and its C2 comes after that -- the Cycle [C2, C1] with V1 under it, in which
    the C1 -> V1 dependency is the one that crosses Cycles (Section 4.1).  With the stage lengths measured on
    the MI355X (cycles per sub-block and wave: C1 36 MFMAs at 32.6 - 37.4, C2 32 MFMAs at 32.6, V1 about 600 of
    vector issue) the rotation rule returns exactly that Cycle, the oracle's timeline admits it, and the vector
    work fits under the matrix work (the theorem's matrix-bound case)."""
    for c1 in (36 * 33, 36 * 37):                 # the first product's MFMAs issue between 32.6 and 37.4 cycles apart
        cube, vec = [c1, 32 * 33], [600, 0]
        assert sum(vec) <= sum(cube)
        first, external, count = amla.amla_preload_rotation(cube, vec)
        assert (first, external, count) == (2, 1, 2)
        assert po.cube_order(2, first) == [2, 1]                 # the Cycle starts with C2 and ends with C1
        assert first in po.admissible_rotations(cube, vec)
    # were the vector stage longer than the matrix stage it hides under plus the slack of the Cycle, no rotation
    # could hide it: the rule refuses the vector-bound case
    with pytest.raises(amla.AmlaError):
        amla.amla_preload_rotation([36 * 33, 32 * 33], [2300, 0])
