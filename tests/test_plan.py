"""The balanced decomposition's integer arithmetic (csrc/amla_plan.h), run on the host through the
C ABI: the same routines the decode and combine kernels use to decide who owns which block."""
import numpy as np
import pytest

from oracle import amla_oracle as orc
from paper_2509_25224_amd import amla


def _cases():
    rng = np.random.default_rng(7)
    yield [4096] * 64, 256
    yield [1, 63, 64, 65, 300, 1000], 8
    yield [0, 0, 5, 0], 3
    yield [70], 5                     # more workers than blocks
    yield [64 * 7] * 3, 7
    for _ in range(40):
        batch = int(rng.integers(1, 40))
        lens = rng.integers(0, 3000, batch)
        lens[rng.random(batch) < 0.15] = 0
        if lens.sum() == 0:
            lens[0] = 1
        yield lens.tolist(), int(rng.integers(1, 300))


@pytest.mark.parametrize("lens,workers", list(_cases()))
def test_pieces_tile_every_sequence_and_agree_with_the_combine_view(lens, workers):
    pieces, seq_workers = amla.amla_plan_segments(lens, workers)
    nb = [(n + 63) // 64 for n in lens]
    total = sum(nb)
    # every block of every sequence exactly once, pieces of a sequence in block order
    covered = {b: [] for b in range(len(lens))}
    for w, b, j0, j1, slot, full in pieces:
        assert 0 <= j0 < j1 <= nb[b]
        assert slot == w + b and 0 <= slot <= workers + len(lens) - 2
        covered[b].append((j0, j1, w, full))
    for b, runs in covered.items():
        at = 0
        for j0, j1, _, _ in runs:
            assert j0 == at
            at = j1
        assert at == nb[b]
        # a piece is full exactly when it is the sequence's only piece
        assert all(full == (len(runs) == 1) for _, _, _, full in runs)
        # what the combine kernel derives: first and last worker, and every worker in between
        # that owns any block has a piece of this sequence
        if nb[b] == 0:
            assert tuple(seq_workers[b]) == (-1, -1)
        else:
            ws = [w for _, _, w, _ in runs]
            assert ws == sorted(ws) and len(set(ws)) == len(ws)
            assert tuple(seq_workers[b]) == (ws[0], ws[-1])
            owning = [w for w in range(ws[0], ws[-1] + 1) if (w * total) // workers < ((w + 1) * total) // workers]
            assert owning == ws
    # slots are unique, pieces come in (worker, sequence) order, shares differ by at most one block
    slots = pieces[:, 4]
    assert np.all(np.diff(slots) > 0)
    share = np.zeros(workers, dtype=np.int64)
    for w, b, j0, j1, slot, full in pieces:
        share[w] += j1 - j0
    assert share.sum() == total and share.max() - share.min() <= 1


def test_merging_the_pieces_gives_the_definition():
    """The scheme itself, in fp64 on the CPU: attention over each piece's keys, merged per sequence
    with weights exp(lse_piece - lse) as the combine kernel does, equals attention over the whole
    sequence."""
    rng = np.random.default_rng(8)
    lens = [130, 0, 700, 64, 1500]
    workers = 6
    pieces, seq_workers = amla.amla_plan_segments(lens, workers)
    for b, n in enumerate(lens):
        if n == 0:
            continue
        Q = rng.standard_normal((4, 576))
        K = rng.standard_normal((n, 576))
        want, want_lse = orc.attention_rows(Q, K, 0.07)
        parts = []
        for w, pb, j0, j1, slot, full in pieces:
            if pb == b:
                parts.append(orc.attention_rows(Q, K[64 * j0:min(n, 64 * j1)], 0.07))
        lses = np.stack([l for _, l in parts])
        mx = lses.max(axis=0)
        wgt = np.exp(lses - mx)
        out = sum(o * w_[:, None] for (o, _), w_ in zip(parts, wgt)) / wgt.sum(axis=0)[:, None]
        assert np.abs(out - want).max() < 1e-12
        assert np.abs(mx + np.log(wgt.sum(axis=0)) - want_lse).max() < 1e-12


def test_plan_rejects_bad_arguments():
    with pytest.raises(amla.AmlaError):
        amla.amla_plan_segments([10, -1], 4)
    with pytest.raises(amla.AmlaError):
        amla.amla_plan_segments([10], 0)
