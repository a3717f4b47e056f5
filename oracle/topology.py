"""Replica-array arithmetic of partial sharding and the peak-memory model.  TEST INFRASTRUCTURE ONLY.

Section 5.1 (multi-phase reduce-scatter on an N x M array of devices: the shard id follows the
topology of all phases), Section 5.2 (partial sharding: the rows of an N x M array of replicas
are independent sharding groups, the columns all-reduce the partial results; a combined all-reduce
partitions the concatenation of its inputs, whatever their individual sharding) and Section 4.2
("Memory saving": peak memory with and without sharded auxiliary variables).

Replica ids are row-major over the array: replica = row * M + column, so the rows of a 2 x 4 array
are {0,1,2,3} and {4,5,6,7} (the all-reduce subgroup example of Section 2.1).

Plain integer arithmetic written from those passages; it shares nothing with the HIP library.
"""
from __future__ import annotations

from fractions import Fraction
from typing import List, Tuple


def _check_array(rows: int, cols: int, replica: int) -> None:
    if rows < 1 or cols < 1:
        raise ValueError("array dimensions must be >= 1")
    if not 0 <= replica < rows * cols:
        raise ValueError("replica id outside the array")


def partial_sharding(rows: int, cols: int, replica: int) -> Tuple[int, int, List[int], List[int]]:
    """Section 5.2.  Returns (group, shard_id, shard_group, reduce_group) of `replica` in a
    rows x cols array: the sharding group is the replica's row (cols members, each owning 1/cols of
    every variable, shard_id = its column), the all-reduce group is its column (rows members, all
    holding the same shard id)."""
    _check_array(rows, cols, replica)
    row, col = divmod(replica, cols)
    shard_group = [row * cols + j for j in range(cols)]
    reduce_group = [i * cols + col for i in range(rows)]
    return row, col, shard_group, reduce_group


def two_phase_shard_id(rows: int, cols: int, replica: int) -> int:
    """Section 5.1.  Full sharding over a rows x cols array in two phases: a reduce-scatter inside
    every row leaves replica (i, j) with piece j of cols pieces; a reduce-scatter inside every
    column then leaves it with sub-piece i of the rows sub-pieces of that piece.  Of the
    rows * cols final pieces, in order of position in the data, that is piece j * rows + i."""
    _check_array(rows, cols, replica)
    i, j = divmod(replica, cols)
    return j * rows + i


def concat_partition(total: int, parts: int, part: int) -> Tuple[int, int]:
    """Section 5.2.  A combined all-reduce sees its inputs concatenated and partitions the
    concatenation into `parts` internal pieces of ceil(total / parts) elements, the last ones
    shorter or empty; no boundary of an input tensor is respected.  Returns (start, length)."""
    if total < 0 or parts < 1 or not 0 <= part < parts:
        raise ValueError("bad partition request")
    piece = -(-total // parts)
    start = min(part * piece, total)
    return start, min(piece, total - start)


def peak_memory(W, V, P, N: int):
    """Section 4.2, "Memory saving".  W: weights, V: auxiliary variables, P: peak of live
    activations and gradients, N: shards.  Returns (replicated, sharded) as exact fractions:
    W + V + P  and  max(W + V/N + P, W + V)."""
    if N < 1 or min(W, V, P) < 0:
        raise ValueError("bad memory model arguments")
    W, V, P = Fraction(W), Fraction(V), Fraction(P)
    return W + V + P, max(W + V / N + P, W + V)


def plan_peak_bytes(numel, S: int, weight_bytes: int, aux_bytes: int, P: int) -> Tuple[int, int]:
    """The same model on a concrete sharding plan, in bytes.  numel: elements of every variable;
    S: packed shard length of the plan (padding included, so V/N becomes S * aux_bytes);
    weight_bytes: bytes per weight element; aux_bytes: bytes of all auxiliary variables per weight
    element (8 for Adam's two float32 moments)."""
    total = sum(int(n) for n in numel)
    W, V = total * weight_bytes, total * aux_bytes
    return W + V + P, max(W + S * aux_bytes + P, W + V)
