"""Oracle of the fragment map and synchronisation schedule (TEST INFRASTRUCTURE ONLY).

Written straight from the definitions, with plain loops:

* Section 2.2 (streaming partial updates): the network's transformer blocks are
  partitioned into P fragments, either *sequential* (consecutive blocks) or
  *strided* (interleaved blocks, the default).
* Algorithm 2, Require list: every fragment p has a synchronisation offset
  t_p; the overlap delay tau is smaller than H.
* Algorithm 2, the two conditions: a fragment's outer gradient is sent when
  (t - t_p) mod H == 0 and the averaged result is received tau steps later.
  Section 2.2 adds that every fragment always does H inner steps before it is
  synchronised, with the worked example H = 100, P = 2: steps 100, 200, ... for
  offset 0 and 150, 250, ... for offset 50.  Hence the first send of fragment
  p is at t_p + H, never at t_p itself.

Readings where the paper is silent: default offsets t_p = floor(p*H/P);
parameters outside the blocks (embedding = UNIT_PRE, head / final norm =
UNIT_POST) travel with the first / last block's fragment; several fragments due
at the same step are all reported, in ascending p.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

PATTERN_STRIDED, PATTERN_SEQUENTIAL = 0, 1
UNIT_PRE, UNIT_POST = -1, -2


@dataclass
class RefPlan:
    P: int
    H: int
    tau: int
    offsets: List[int]
    block_fragment: List[int]                       # fragment of each transformer block
    spans: List[List[Tuple[int, int, int]]] = field(default_factory=list)  # per p: (offset, numel, unit)
    total: int = 0

    def sends(self, t: int) -> List[int]:
        out = []
        for p in range(self.P):
            k = 1
            while self.offsets[p] + k * self.H <= t:
                if self.offsets[p] + k * self.H == t:
                    out.append(p)
                k += 1
        return out

    def receives(self, t: int) -> List[int]:
        out = []
        for p in range(self.P):
            k = 1
            while self.offsets[p] + k * self.H + self.tau <= t:
                if self.offsets[p] + k * self.H + self.tau == t:
                    out.append(p)
                k += 1
        return out


def fragment_plan(unit_numel: Sequence[int], unit_block: Sequence[int], n_blocks: int, P: int,
                  pattern: int, H: int, tau: int, t_p: Optional[Sequence[int]] = None,
                  pre_own_fragment: bool = False, align: int = 1) -> RefPlan:
    """pre_own_fragment: the embedding (UNIT_PRE) is a fragment of its own, number 0, and the
    blocks use fragments 1..P -- the reading under which the appendix's "8, 16, 36 fragments,
    one synchronised every 11, 5, 2 steps" adds up (H / (fragments + 1)).

    align: a memory-layout option, not part of the method: every parameter group starts at the
    next multiple of `align` elements; the padding in between belongs to no fragment."""
    assert 1 <= P <= n_blocks and H >= 1 and 0 <= tau < H
    shift = 1 if pre_own_fragment else 0
    block_fragment = []
    for i in range(n_blocks):
        if pattern == PATTERN_STRIDED:
            block_fragment.append(shift + i % P)
        else:
            owner = None
            for p in range(P):
                if (p * n_blocks) // P <= i < ((p + 1) * n_blocks) // P:
                    owner = p
            block_fragment.append(shift + owner)
    P = P + shift
    offsets = [(p * H) // P for p in range(P)] if t_p is None else [int(x) for x in t_p]
    spans = [[] for _ in range(P)]
    pos = 0
    for u, (numel, blk) in enumerate(zip(unit_numel, unit_block)):
        while pos % align != 0:
            pos += 1
        if blk == UNIT_PRE:
            p = 0 if pre_own_fragment else block_fragment[0]
        elif blk == UNIT_POST:
            p = block_fragment[n_blocks - 1]
        else:
            assert 0 <= blk < n_blocks
            p = block_fragment[blk]
        spans[p].append((pos, int(numel), u))
        pos += int(numel)
    return RefPlan(P=P, H=H, tau=tau, offsets=offsets, block_fragment=block_fragment, spans=spans,
                   total=pos)
