"""Pins of the Preload Pipeline oracle (oracle/preload_oracle.py): the timeline definition of an
admissible Cycle rotation against what the paper prints (Section 4.1; Appendix B: Lemma B.1, the three
compound conditions for n = 3, the compound inequality of Theorem B.3, the existence claim)."""
import itertools
import os
import random
import sys

import pytest

sys.path.insert(0, os.path.join(os.path.dirname(__file__), "..", "oracle"))
import preload_oracle as po  # noqa: E402


def _durations(rng, n, cube_bound=True):
    while True:
        cube = [rng.randint(0, 40) for _ in range(n)]
        vec = [rng.randint(0, 40) for _ in range(n)]
        if not cube_bound or sum(vec) <= sum(cube):
            return cube, vec


def test_the_three_conditions_printed_for_n_3():
    """Appendix B lists, for the clockwise permutations C1C2C3, C2C3C1, C3C1C2, the conditions under
    which two C -> V chains stay inside the Cycle."""
    rng = random.Random(1)
    seen = set()
    for _ in range(4000):
        (c1, c2, c3), (v1, v2, v3) = _durations(rng, 3, cube_bound=False)
        printed = {1: v1 + v2 <= c2 + c3 and v2 <= c3,
                   2: v2 + v3 <= c3 + c1 and v3 <= c1,
                   3: v3 + v1 <= c1 + c2 and v1 <= c2}
        for s in (1, 2, 3):
            assert po.admissible((c1, c2, c3), (v1, v2, v3), s) == printed[s]
            seen.add((s, printed[s]))
    assert len(seen) == 6                                   # both outcomes of every condition occurred


def _theorem_b3(cube, vec, k):
    """The compound inequality of Theorem B.3 for index k, with the paper's cyclic indexing."""
    n = len(cube)
    C = lambda i: cube[(i - 1) % n]                         # noqa: E731  (1-based, cyclic)
    V = lambda i: vec[(i - 1) % n]                          # noqa: E731
    return all(sum(V(n - k - i) for i in range(j)) <= sum(C(n + 1 - k - i) for i in range(j))
               for j in range(1, n))


@pytest.mark.parametrize("n", [2, 3, 4, 5, 7])
def test_timeline_equals_the_compound_inequality(n):
    """Index k of Theorem B.3 is the Cycle whose last Cube stage is C_{n+1-k}, i.e. that starts with
    C_{n+2-k}."""
    rng = random.Random(n)
    outcomes = set()
    for _ in range(1500):
        cube, vec = _durations(rng, n, cube_bound=False)
        for k in range(1, n + 1):
            s = (n + 1 - k) % n + 1
            assert po.cube_order(n, s)[-1] == (n - k) % n + 1
            got = po.admissible(cube, vec, s)
            assert got == _theorem_b3(cube, vec, k)
            outcomes.add(got)
    assert outcomes == {True, False}


@pytest.mark.parametrize("n", [1, 2, 3, 4, 6, 8])
def test_existence_when_the_cube_stages_dominate(n):
    """Theorem B.3 / Theorem 4.1: sum V <= sum C guarantees an admissible rotation, whatever the split."""
    rng = random.Random(100 + n)
    for trial in range(3000):
        cube, vec = _durations(rng, n)
        if trial % 3 == 0 and n > 1:                        # one Vector stage takes all of the budget
            k = rng.randrange(n)
            vec = [0] * n
            vec[k] = sum(cube)
        assert po.admissible_rotations(cube, vec)


def test_without_the_condition_no_rotation_need_exist():
    assert po.admissible_rotations([1, 1, 1], [5, 5, 5]) == []


def test_exhaustive_small_case_against_all_orders():
    """Brute force on tiny inputs: try every start of the Vector stages on an integer grid instead of
    the greedy timeline; the chained stages fit into the Cycle exactly when the timeline says so."""
    for cube in itertools.product(range(0, 4), repeat=2):
        for vec in itertools.product(range(0, 5), repeat=2):
            for s in (1, 2):
                order = po.cube_order(2, s)
                i = order[0]                                # the one chained pair for n = 2
                end_c = cube[i - 1]
                fits = any(start >= end_c and start + vec[i - 1] <= sum(cube) for start in range(0, sum(cube) + 1))
                assert po.admissible(cube, vec, s) == fits


def test_amla_chain_has_the_cycle_of_section_4_1():
    """n = 2 with V2 = 0: the Cycle [.., C2, C1] (the paper writes it [C1, C2, V1]: V1 takes C1's result
    of the previous Cycle) is admissible whatever the three durations; Preload count 2."""
    rng = random.Random(7)
    for _ in range(500):
        c1, c2, v1 = rng.randint(0, 50), rng.randint(0, 50), rng.randint(0, 50)
        assert po.admissible((c1, c2), (v1, 0), 2)
        assert po.admissible((c1, c2), (v1, 0), 1) == (v1 <= c2)
    assert po.preload_count(2, 1) == 2


def test_lemma_b1_counts():
    for n in range(1, 9):
        assert po.preload_count(n, 0) == 2 * n - 1          # nothing chained: the whole chain is preloaded
        assert po.preload_count(n, n - 1) == n              # the bound of Theorem 4.1
