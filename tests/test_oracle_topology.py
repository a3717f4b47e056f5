"""Pins for oracle/topology.py: the replica-array examples the paper states, brute-force
simulations of the collectives on tiny arrays, closed forms of the memory model."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import make_plan
from oracle.topology import (concat_partition, partial_sharding, peak_memory, plan_peak_bytes,
                             two_phase_shard_id)
from workloads import CONFIGS

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "topology_examples.txt")


def _golden(kind):
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            parts = line.split()
            if parts and parts[0] == kind:
                rows.append(tuple(int(x) for x in parts[1:]))
    assert rows
    return rows


@pytest.mark.parametrize("row", _golden("rowgroup"))
def test_papers_subgroup_example(row):
    rows, cols, which, members = row[0], row[1], row[2], list(row[3:])
    for replica in members:
        group, shard_id, shard_group, _ = partial_sharding(rows, cols, replica)
        assert group == which and shard_group == members and members[shard_id] == replica


@pytest.mark.parametrize("replicas,group_size,n_groups", _golden("groups"))
def test_papers_pod_example(replicas, group_size, n_groups):
    rows, cols = replicas // group_size, group_size
    assert rows == n_groups
    seen_groups = {}
    for replica in range(replicas):
        group, shard_id, shard_group, reduce_group = partial_sharding(rows, cols, replica)
        assert len(shard_group) == group_size and len(reduce_group) == n_groups
        assert 0 <= shard_id < group_size
        seen_groups.setdefault(group, set()).add(replica)
    assert len(seen_groups) == n_groups and all(len(s) == group_size for s in seen_groups.values())


@pytest.mark.parametrize("rows,cols", [(1, 1), (1, 5), (5, 1), (2, 4), (3, 3), (4, 6)])
def test_partial_sharding_equals_the_full_all_reduce_piece(rows, cols):
    # Section 5.2 by brute force: a reduce-scatter inside every sharding group followed by an
    # all-reduce over every reduce group leaves each replica with its piece of the sum over ALL replicas.
    rng = np.random.default_rng(rows * 10 + cols)
    R, piece = rows * cols, 3
    grads = rng.integers(-50, 50, size=(R, cols * piece)).astype(np.int64)     # integers: sums are exact
    total = grads.sum(axis=0)
    info = [partial_sharding(rows, cols, q) for q in range(R)]
    after_rs = []
    for q in range(R):
        _, sid, sgroup, _ = info[q]
        after_rs.append(sum(grads[p][sid * piece:(sid + 1) * piece] for p in sgroup))
    for q in range(R):
        _, sid, sgroup, rgroup = info[q]
        got = sum(after_rs[p] for p in rgroup)
        assert np.array_equal(got, total[sid * piece:(sid + 1) * piece])
        # every member of the reduce group holds the same shard id, every member of the shard group a different one
        assert {info[p][1] for p in rgroup} == {sid}
        assert sorted(info[p][1] for p in sgroup) == list(range(cols))
    # the groups partition the replicas both ways
    assert sorted(q for g in {tuple(i[2]) for i in info} for q in g) == list(range(R))
    assert sorted(q for g in {tuple(i[3]) for i in info} for q in g) == list(range(R))


@pytest.mark.parametrize("rows,cols", [(1, 1), (1, 4), (4, 1), (2, 3), (3, 2), (4, 4), (3, 5)])
def test_two_phase_shard_id_by_simulation(rows, cols):
    # Section 5.1 by brute force: row phase, then column phase, on integer data.
    rng = np.random.default_rng(100 + rows * 10 + cols)
    R, sub = rows * cols, 2
    D = R * sub
    data = rng.integers(-50, 50, size=(R, D)).astype(np.int64)
    total = data.sum(axis=0)
    big = D // cols
    phase1 = {}
    for i in range(rows):
        for j in range(cols):
            phase1[(i, j)] = sum(data[i * cols + jj][j * big:(j + 1) * big] for jj in range(cols))
    ids = []
    for i in range(rows):
        for j in range(cols):
            mine = sum(phase1[(ii, j)][i * sub:(i + 1) * sub] for ii in range(rows))
            sid = two_phase_shard_id(rows, cols, i * cols + j)
            assert np.array_equal(mine, total[sid * sub:(sid + 1) * sub])
            ids.append(sid)
    assert sorted(ids) == list(range(R))


@pytest.mark.parametrize("N,M,D,size1,size2", _golden("phases"))
def test_papers_phase_sizes(N, M, D, size1, size2):
    assert make_plan([D], M, 1).L[0] == size1                 # first phase: M pieces of D/M
    assert make_plan([size1], N, 1).L[0] == size2             # second phase: N pieces of D/(M*N)
    assert make_plan([D], M * N, 1).L[0] == size2             # the same pieces as one-phase sharding N*M ways
    ids = sorted(two_phase_shard_id(N, M, q) for q in range(N * M))
    assert ids == list(range(N * M))


def test_degenerate_arrays():
    for q in range(7):
        assert two_phase_shard_id(1, 7, q) == q               # one row: the shard id is the column
        assert two_phase_shard_id(7, 1, q) == q               # one column: it is the row
        assert partial_sharding(1, 7, q)[:2] == (0, q) and partial_sharding(1, 7, q)[3] == [q]
        assert partial_sharding(7, 1, q)[:2] == (q, 0) and partial_sharding(7, 1, q)[2] == [q]
    with pytest.raises(ValueError):
        partial_sharding(2, 2, 4)
    with pytest.raises(ValueError):
        two_phase_shard_id(0, 2, 0)


@pytest.mark.parametrize("total,parts", [(0, 1), (0, 3), (1, 4), (10, 3), (12, 4), (13, 4), (1000, 7), (5, 8)])
def test_concat_partition_tiles_the_concatenation(total, parts):
    pos = 0
    for k in range(parts):
        start, length = concat_partition(total, parts, k)
        assert start == pos and 0 <= length <= -(-total // parts)
        pos += length
    assert pos == total
    if total % parts == 0 and total > 0:                      # equal pieces: numpy's split boundaries
        pieces = np.split(np.arange(total), parts)
        for k in range(parts):
            start, length = concat_partition(total, parts, k)
            assert (pieces[k][0], len(pieces[k])) == (start, length)


def test_combined_all_reduce_ignores_tensor_boundaries():
    # Section 5.2: the inputs are concatenated in full shapes; internal pieces are cut on the concatenation.
    sizes = [5, 1, 7, 2]
    flat = np.concatenate([np.full(n, i) for i, n in enumerate(sizes)])
    start, length = concat_partition(len(flat), 3, 1)
    assert (start, length) == (5, 5)
    assert set(flat[start:start + length]) == {1, 2}            # one piece spans tensors 1 and 2


@pytest.mark.parametrize("W,V,P,N,rep,sh", _golden("memory"))
def test_memory_model_hand_worked(W, V, P, N, rep, sh):
    assert peak_memory(W, V, P, N) == (rep, sh)


def test_memory_model_properties():
    W, V, P = 340, 680, 500                                     # Adam: V = 2W
    rep, one = peak_memory(W, V, P, 1)
    assert rep == one == W + V + P                              # one shard: nothing saved
    prev = one
    for N in (2, 4, 8, 64, 2048):
        rep, sh = peak_memory(W, V, P, N)
        assert rep == W + V + P and W + V <= sh <= prev         # never below the out-of-loop footprint
        assert sh == max(Fraction(W) + Fraction(V, N) + P, W + V)
        prev = sh
    # Section 4.2: with enough shards Adam's peak approaches SGD's (V = 0) when activations dominate
    sgd = peak_memory(W, 0, 2000, 64)[1]
    adam = peak_memory(W, V, 2000, 64)[1]
    assert sgd == W + 2000 and adam - sgd == Fraction(V, 64)
    with pytest.raises(ValueError):
        peak_memory(1, 1, 1, 0)


def test_plan_peak_bytes_matches_the_model_when_nothing_is_padded():
    cfg = [c for c in CONFIGS if c.name == "transformer_big"][0]       # every variable divides by 16 * 8
    numel = list(cfg.numel)
    plan = make_plan(numel, 16, 8)
    assert plan.S * 16 == sum(numel)
    P = 10 ** 9
    rep, sh = plan_peak_bytes(numel, plan.S, 4, 8, P)
    W, V = 4 * sum(numel), 8 * sum(numel)
    assert (rep, sh) == peak_memory(W, V, P, 16)
    # with padding the sharded auxiliaries cost S, not total/N
    numel = [10, 3]
    plan = make_plan(numel, 4, 8)
    assert plan_peak_bytes(numel, plan.S, 4, 8, 1000) == (13 * 12 + 1000, max(13 * 4 + 16 * 8 + 1000, 13 * 12))
