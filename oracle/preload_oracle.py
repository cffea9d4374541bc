"""CPU oracle for the Preload Pipeline's Cycle rotation.  TEST INFRASTRUCTURE ONLY.

Shares no code with the library; only tests call it.

Setting (Section 4.1, Appendix B): one Cycle of the steady loop runs the n Cube stages C_1 .. C_n of
the chain C_1 -> V_1 -> C_2 -> ... -> C_n -> V_n back to back in some cyclic order, so a Cycle lasts
sum(C).  A dependency C_i -> V_i kept *inside* the Cycle saves one preloaded stage (Lemma B.1:
Preload count = (2n - 1) - s for s internal chains); every V_i -> C_{i+1} edge crosses Cycles.  With
the Cube order C_s, C_{s+1}, .., C_{s+n-1} (indices cyclic) the n - 1 pairs that can be chained are
those of every Cube stage but the last one.

`admissible(cube, vec, s)` is the definition written out as a timeline: the Vector unit takes the
chained stages in order, each starting when its Cube stage and the previous Vector stage are done,
and the rotation is admissible when the last of them ends no later than the Cycle.  This is what
the compound inequality of Theorem B.3 states in closed form (pinned against the three conditions
the paper prints for n = 3, and against the inequality itself).

`admissible_rotations` lists every admissible first stage s in 1..n by trying them all.
"""
from __future__ import annotations


def cube_order(n: int, s: int) -> list[int]:
    """Stage numbers (1-based) of the Cycle that starts with C_s."""
    return [(s - 1 + i) % n + 1 for i in range(n)]


def admissible(cube, vec, s: int) -> bool:
    """Timeline check of the Cycle starting with C_s (1-based), durations as sequences of length n."""
    n = len(cube)
    order = cube_order(n, s)
    cycle = float(sum(cube))
    t_cube = 0.0
    t_vec = 0.0
    for pos, i in enumerate(order):
        t_cube += cube[i - 1]                      # C_i ends
        if pos < n - 1:                            # V_i is chained behind it inside the Cycle
            t_vec = max(t_vec, t_cube) + vec[i - 1]
    return t_vec <= cycle


def admissible_rotations(cube, vec) -> list[int]:
    return [s for s in range(1, len(cube) + 1) if admissible(cube, vec, s)]


def preload_count(n: int, internal_chains: int) -> int:
    """Lemma B.1."""
    return (2 * n - 1) - internal_chains
