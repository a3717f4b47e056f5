"""Sharding representation of a list of variables (Section 4.1, "Data formatting").

Each variable is flattened (a reshape that moves no data in linear row-major
memory), padded at its tail until N equal pieces fit, and replica r owns the
piece that starts at r times the piece length (the dynamic-slice whose offset
is computed from the replica id).  A replica's packed shard holds one piece of
every variable, in the caller's variable order (Section 5.2, "Batched
communication operators").  `align` stands in for the hardware access granule
(the paper's platform-dependent bitcast serves the same purpose on TPU tiles);
align = 1 is the bare ceil(n / N) rule.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence


@dataclass(frozen=True)
class Plan:
    numel: tuple   # n_i
    N: int
    align: int
    L: tuple       # piece length of variable i, the same on every replica
    off: tuple     # offset of variable i's piece inside a packed shard
    S: int         # packed shard length

    @property
    def V(self) -> int:
        return len(self.numel)

    def real_count(self, i: int, r: int) -> int:
        """How many of replica r's L_i slots of variable i hold real (unpadded) elements."""
        start = r * self.L[i]
        return max(0, min(self.L[i], self.numel[i] - start))


def make_plan(numel: Sequence[int], N: int, align: int = 8) -> Plan:
    if N < 1:
        raise ValueError("replica count must be >= 1")
    if align < 1 or (align & (align - 1)) != 0:
        raise ValueError("align must be a power of two")
    L: List[int] = []
    off: List[int] = []
    pos = 0
    for n in numel:
        n = int(n)
        if n < 0:
            raise ValueError("negative element count")
        per_replica = -(-n // N)                         # ceil(n / N)
        length = -(-per_replica // align) * align        # rounded up to the granule
        L.append(length)
        off.append(pos)
        pos += length
    return Plan(tuple(int(n) for n in numel), int(N), int(align), tuple(L), tuple(off), pos)
