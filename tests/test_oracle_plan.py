"""Pins of the oracle's fragment map and schedule against the paper's worked example,
its stated invariants and counting arguments."""
import os

import pytest

import workloads
from oracle import PATTERN_SEQUENTIAL, PATTERN_STRIDED, fragment_plan

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    return [l.split() for l in open(os.path.join(GOLDEN, name)) if l.strip() and not l.startswith("#")]


def _blocks_only(L, numel=10):
    return [numel] * L, list(range(L))


def test_worked_example_section_2_2():
    for H, P, p, off, *steps in _rows("schedule_example.txt"):
        H, P, p, off = int(H), int(P), int(p), int(off)
        plan = fragment_plan(*_blocks_only(4), 4, P, PATTERN_STRIDED, H, 0)
        assert plan.offsets[p] == off
        got = [t for t in range(1, 460) if p in plan.sends(t)]
        assert got == [int(s) for s in steps]


@pytest.mark.parametrize("P,H,tau", [(1, 100, 0), (2, 100, 1), (3, 100, 1), (4, 100, 5), (6, 100, 1),
                                     (8, 100, 20), (5, 7, 6)])
def test_every_fragment_does_H_steps_before_sync(P, H, tau):
    plan = fragment_plan(*_blocks_only(8), 8, P, PATTERN_STRIDED, H, tau)
    T = 3 * H + tau + H
    for p in range(P):
        sends = [t for t in range(1, T + 1) if p in plan.sends(t)]
        recvs = [t for t in range(1, T + 1) if p in plan.receives(t)]
        assert sends[0] == plan.offsets[p] + H >= H
        assert all(b - a == H for a, b in zip(sends, sends[1:]))
        assert len(sends) == (T - plan.offsets[p]) // H          # closed-form count
        assert recvs == [t + tau for t in sends if t + tau <= T]
        # Algorithm 2's conditions hold at every reported step
        assert all((t - plan.offsets[p]) % H == 0 for t in sends)
        assert all((t - plan.offsets[p] - tau) % H == 0 for t in recvs)


def test_fragment_counts_and_peak_factor():
    for L, per, P, _every in _rows("fragment_counts.txt"):
        L, per, P = int(L), int(per), int(P)
        assert L // per == P
        for pattern in (PATTERN_STRIDED, PATTERN_SEQUENTIAL):
            plan = fragment_plan(*_blocks_only(L), L, P, pattern, 100, 1)
            sizes = [sum(n for _, n, _ in plan.spans[p]) for p in range(P)]
            assert sizes == [per * 10] * P                      # |p| / L of the model each
            assert max(sizes) * P == plan.total


def test_patterns():
    strided = fragment_plan(*_blocks_only(12), 12, 3, PATTERN_STRIDED, 100, 1)
    assert strided.block_fragment == [0, 1, 2] * 4
    seq = fragment_plan(*_blocks_only(12), 12, 3, PATTERN_SEQUENTIAL, 100, 1)
    assert seq.block_fragment == [0] * 4 + [1] * 4 + [2] * 4
    uneven = fragment_plan(*_blocks_only(7), 7, 3, PATTERN_SEQUENTIAL, 100, 1)
    assert uneven.block_fragment == [0, 0, 1, 1, 2, 2, 2]
    assert sorted(set(uneven.block_fragment)) == [0, 1, 2]


@pytest.mark.parametrize("name,P,sizes,total", [
    ("100m", 3, [52893696, 28317696, 52894464], 134105856),
    ("1b", 4, [367550464, 302014464, 302014464, 367552512], 1339131904),
    ("4b", 6, [777818112] + [679514112] * 4 + [777821184], 4273695744),
    ("4b", 1, [4273695744], 4273695744),
])
def test_decoder_shapes_partition_exactly(name, P, sizes, total):
    numel, block, _ = workloads.SHAPES[name].units()
    L = workloads.SHAPES[name].n_layers
    plan = fragment_plan(numel, block, L, P, PATTERN_STRIDED, 100, 1)
    assert plan.total == total == sum(numel)
    assert [sum(n for _, n, _ in plan.spans[p]) for p in range(P)] == sizes
    assert plan.offsets == [(p * 100) // P for p in range(P)]
    # spans tile [0, total) exactly once
    allspans = sorted(s for p in range(P) for s in plan.spans[p])
    pos = 0
    for off, n, _ in allspans:
        assert off == pos
        pos += n
    assert pos == total
    assert all(n % 32 == 0 for _, n, _ in allspans)


def test_aligned_layout_pads_to_the_next_boundary_and_no_further():
    """The layout option moves nothing between fragments; every group starts on a multiple of the
    alignment, directly behind its predecessor's last element rounded up, and the sizes are kept."""
    numel = [5, 64, 0, 63, 65, 128, 1, 1, 200]
    block = [-1, 0, 0, 1, 1, 2, 2, -2, -2]
    plain = fragment_plan(numel, block, 3, 3, PATTERN_STRIDED, 10, 1)
    padded = fragment_plan(numel, block, 3, 3, PATTERN_STRIDED, 10, 1, align=64)
    assert [[(n, u) for _, n, u in f] for f in padded.spans] == [[(n, u) for _, n, u in f] for f in plain.spans]
    by_unit = sorted((u, off, n) for f in padded.spans for off, n, u in f)
    assert [off for _, off, _ in by_unit] == [0, 64, 128, 128, 192, 320, 448, 512, 576]   # worked by hand
    assert padded.total == 576 + 200 and plain.total == sum(numel)
    assert fragment_plan(numel, block, 3, 3, PATTERN_STRIDED, 10, 1, align=1).spans == plain.spans


def test_colliding_offsets_all_reported():
    plan = fragment_plan(*_blocks_only(4), 4, 4, PATTERN_STRIDED, 100, 30, t_p=[0, 0, 30, 60])
    assert plan.sends(100) == [0, 1]
    assert plan.sends(130) == [2] and plan.receives(130) == [0, 1]
    assert plan.receives(160) == [2] and plan.sends(160) == [3]


def test_embedding_as_its_own_fragment_reproduces_the_appendix_counts():
    """Appendix (compute utilisation): 3 layers per fragment -> 8 / 16 / 36 fragments for 24 / 48 /
    108 layers, and some fragment is synchronised every 11 / 5 / 2 steps with H = 100.  The step
    counts only add up with one more fragment (the embedding): floor(100 / (fragments + 1))."""
    for L, per, P, every in _rows("fragment_counts.txt"):
        L, per, P, every = int(L), int(per), int(P), int(every)
        numel = [1000] + [10] * L + [5, 1000]
        block = [-1] + list(range(L)) + [-2, -2]
        assert 100 // (P + 1) == every
        offs = [p * every for p in range(P + 1)]
        plan = fragment_plan(numel, block, L, P, PATTERN_STRIDED, 100, 1, t_p=offs, pre_own_fragment=True)
        assert plan.P == P + 1
        assert plan.spans[0] == [(0, 1000, 0)]                              # the embedding alone
        assert all(len([b for b in plan.block_fragment if b == p]) == per for p in range(1, P + 1))
        syncs = sorted(t for t in range(100, 200) for _ in plan.sends(t))     # one period
        gaps = [b - a for a, b in zip(syncs, syncs[1:])]
        assert len(syncs) == P + 1 and set(gaps) == {every}
