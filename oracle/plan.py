"""Sharding representation of a list of variables (Section 4.1, "Data formatting").

Flat plan (make_plan).  Each variable is flattened (a reshape that moves no data in linear
row-major memory), padded at its tail until N equal pieces fit, and replica r owns the piece that
starts at r times the piece length (the dynamic-slice whose offset is computed from the replica
id).  `align` stands in for the hardware access granule (the paper's platform-dependent bitcast
serves the same purpose on TPU tiles); align = 1 is the bare ceil(n / N) rule.

Row plan (make_row_plan).  The paper's own format: the leading dimensions are combined into one
row dimension, that dimension is padded to a multiple of N and sliced, and the trailing dimensions
stay whole, e.g. [3,3,256,256] -> [9,256,256] -> [10,256,256] at 10 replicas.  A reshape must not
merge a dimension a reduce collapses with one it keeps (Section 4.1, "Non-elementwise operators"),
so optimizers that reduce along rows or columns need this plan.  Replica r owns rows
[r*Lr, (r+1)*Lr) with Lr = ceil(rows / N); its piece holds Lr*cols slots, rounded up to `align`.

In both plans a replica's packed shard holds one piece of every variable, in the caller's variable
order (Section 5.2, "Batched communication operators").
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence, Tuple


@dataclass(frozen=True)
class Plan:
    numel: tuple   # n_i
    N: int
    align: int
    L: tuple       # slots of variable i in every replica's shard
    off: tuple     # offset of variable i's piece inside a packed shard
    S: int         # packed shard length
    stride: tuple  # distance, in the flat variable, between the pieces of consecutive replicas (<= L)
    rows: tuple = None   # row plan only: rows_i, cols_i, and rows per replica Lr_i
    cols: tuple = None
    Lr: tuple = None

    @property
    def V(self) -> int:
        return len(self.numel)

    def real_count(self, i: int, r: int) -> int:
        """How many of replica r's L_i slots of variable i hold real (unpadded) elements."""
        start = r * self.stride[i]
        return max(0, min(self.stride[i], self.numel[i] - start))

    def real_rows(self, i: int, r: int) -> int:
        """Row plan: how many of replica r's Lr_i rows of variable i exist."""
        return max(0, min(self.Lr[i], self.rows[i] - r * self.Lr[i]))


def _check(N: int, align: int) -> None:
    if N < 1:
        raise ValueError("replica count must be >= 1")
    if align < 1 or (align & (align - 1)) != 0:
        raise ValueError("align must be a power of two")


def make_plan(numel: Sequence[int], N: int, align: int = 8) -> Plan:
    _check(N, align)
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
    return Plan(tuple(int(n) for n in numel), int(N), int(align), tuple(L), tuple(off), pos, tuple(L))


def make_row_plan(shapes: Sequence[Tuple[int, int]], N: int, align: int = 8) -> Plan:
    """shapes[i] = (rows_i, cols_i): the variable seen as a row-major matrix; rows are sharded."""
    _check(N, align)
    numel, L, off, stride, rows, cols, Lr = [], [], [], [], [], [], []
    pos = 0
    for (r_i, c_i) in shapes:
        r_i, c_i = int(r_i), int(c_i)
        if r_i < 0 or c_i < 0:
            raise ValueError("negative dimension")
        rows_per_replica = -(-r_i // N) if c_i > 0 else 0
        piece = rows_per_replica * c_i                   # whole rows only
        length = -(-piece // align) * align
        numel.append(r_i * c_i); rows.append(r_i); cols.append(c_i); Lr.append(rows_per_replica)
        L.append(length); stride.append(piece); off.append(pos)
        pos += length
    return Plan(tuple(numel), int(N), int(align), tuple(L), tuple(off), pos, tuple(stride),
                tuple(rows), tuple(cols), tuple(Lr))
