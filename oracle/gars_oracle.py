"""CPU oracle for graph-aware rescheduling (paper, Appendix A.2, Algorithm 1).  TEST
INFRASTRUCTURE ONLY: plain Python loops in the algorithm's order -- sort the global batch by
atom count (descending), give each graph to the micro-batch whose total size is currently the
smallest, shuffle every micro-batch, tag it comm_free iff its largest graph is at most the
per-rank budget sum/d_gp, else dist.  Shares no code with the library's routine.

Readings where the paper is silent: equal sizes keep their original order; equal loads pick
the lowest micro-batch index; the shuffle is Fisher-Yates from the last position down with a
counter-based generator (splitmix64 finaliser; stream = micro-batch index, counter = position),
which the library implements too so that the two can be compared draw for draw.

Pins (tests/test_next_items.py): every graph placed exactly once; max load - min load <= the
largest graph (property of longest-first placement); makespan within 4/3 - 1/(3m) of the
brute-force optimum on tiny instances (the textbook bound); tags against a direct evaluation of
the rule; a worked example done by hand."""
from __future__ import annotations

from typing import List, Tuple

M64 = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15


def _mix(z: int) -> int:
    z &= M64
    z ^= z >> 30
    z = (z * 0xBF58476D1CE4E5B9) & M64
    z ^= z >> 27
    z = (z * 0x94D049BB133111EB) & M64
    z ^= z >> 31
    return z


def _draw(seed: int, stream: int, counter: int) -> int:
    key = _mix(seed ^ ((stream * GOLDEN) & M64))
    return _mix((key + (counter + 1) * GOLDEN) & M64)


def gars_pack(sizes: List[int], n_mb: int, d_gp: int, seed: int) -> Tuple[List[List[int]], List[str]]:
    """Returns (micro-batches as lists of graph indices in shuffled order, tags)."""
    order = sorted(range(len(sizes)), key=lambda g: (-sizes[g], g))
    mbs: List[List[int]] = [[] for _ in range(n_mb)]
    loads = [0] * n_mb
    for g in order:
        j = min(range(n_mb), key=lambda q: (loads[q], q))
        mbs[j].append(g)
        loads[j] += sizes[g]
    tags = []
    for j, mb in enumerate(mbs):
        for t in range(len(mb) - 1, 0, -1):
            r = _draw(seed, j, t) % (t + 1)
            mb[t], mb[r] = mb[r], mb[t]
        c_rank = sum(sizes[g] for g in mb) / d_gp
        biggest = max((sizes[g] for g in mb), default=0)
        tags.append("comm_free" if biggest <= c_rank else "dist")
    return mbs, tags
