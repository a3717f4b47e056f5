"""Pins for the row-granular plan (the paper's own format) and for formatting / reductions on it."""
import os
import random

import numpy as np
import pytest

from oracle import (make_plan, make_row_plan, shard_format, unshard_format, lamb_unsharded_step,
                    lamb_shard_partials, lamb_shard_apply, adam_step)
from workloads import normal_f32, random_bits_u32

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "row_plan_examples.txt")
LAMB = {"lr": 1e-3, "beta1": 0.9, "beta2": 0.999, "eps": 1e-6, "weight_decay": 0.01}


def _rows():
    with open(GOLDEN) as f:
        return [tuple(int(x) for x in l.split()) for l in f if l.strip() and not l.startswith("#")]


@pytest.mark.parametrize("rows,cols,N,per,padded,pad_elems", _rows())
def test_paper_row_format_examples(rows, cols, N, per, padded, pad_elems):
    p = make_row_plan([(rows, cols)], N, 1)
    assert p.Lr[0] == per and p.Lr[0] * N == padded
    assert N * p.S - rows * cols == pad_elems
    assert p.stride[0] == per * cols and p.L[0] == p.stride[0]


def test_alternatives_the_paper_rejects_pad_more():
    # padding [3,3,...] to [10,3,...] or [4,5,...] instead of combining the leading dims first
    combined = make_row_plan([(9, 65536)], 10, 1)
    assert 10 * combined.S == 10 * 65536 < 20 * 65536 < 30 * 65536


def test_row_plan_invariants_and_whole_rows():
    rnd = random.Random(5)
    for _ in range(60):
        N = rnd.randint(1, 40)
        align = rnd.choice([1, 4, 8])
        shapes = [(rnd.choice([0, 1, 2, 3, 7, 9, N - 1, N, N + 1, 100]), rnd.choice([1, 3, 8, 10, 64, 100])) for _ in range(6)]
        p = make_row_plan(shapes, N, align)
        assert p.S == sum(p.L)
        for i, (rows, cols) in enumerate(shapes):
            assert p.numel[i] == rows * cols and p.L[i] % align == 0
            assert p.stride[i] == p.Lr[i] * cols <= p.L[i] < p.stride[i] + align
            assert N * p.Lr[i] >= rows and (p.Lr[i] == 0 or N * (p.Lr[i] - 1) < rows)
            assert sum(p.real_count(i, r) for r in range(N)) == rows * cols
            assert sum(p.real_rows(i, r) for r in range(N)) == rows
            for r in range(N):
                assert p.real_count(i, r) == p.real_rows(i, r) * cols        # a replica never holds part of a row


def test_one_column_row_plan_is_the_flat_plan_when_no_alignment_is_asked():
    numel = [10, 1, 0, 7, 1001]
    a, b = make_plan(numel, 3, 1), make_row_plan([(n, 1) for n in numel], 3, 1)
    assert (a.L, a.off, a.S, a.stride) == (b.L, b.off, b.S, b.stride)


def test_row_plan_format_against_matrix_slicing():
    """Replica r's piece is rows [r*Lr, (r+1)*Lr) of the matrix, zero rows after the last real one."""
    shapes = [(9, 16), (5, 3), (1, 7), (0, 4), (12, 10)]
    N = 4
    p = make_row_plan(shapes, N, 8)
    mats = [random_bits_u32(3, i, r * c).view(np.float32).reshape(r, c) for i, (r, c) in enumerate(shapes)]
    flats = [m.ravel() for m in mats]
    for r in range(N):
        s = shard_format(p, r, flats).view(np.uint32)
        for i, (rows, cols) in enumerate(shapes):
            piece = np.zeros((p.Lr[i], cols), np.uint32)
            lo, hi = r * p.Lr[i], min(rows, (r + 1) * p.Lr[i])
            if hi > lo:
                piece[:hi - lo] = mats[i].view(np.uint32)[lo:hi]
            want = np.zeros(p.L[i], np.uint32)
            want[:piece.size] = piece.ravel()
            assert np.array_equal(s[p.off[i]:p.off[i] + p.L[i]], want)
    gathered = np.stack([shard_format(p, r, flats) for r in range(N)])
    for a, b in zip(flats, unshard_format(p, gathered)):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_row_plan_round_trip_random():
    rnd = random.Random(9)
    for N in (1, 2, 3, 7, 8, 33):
        shapes = [(rnd.choice([0, 1, 5, N, N + 1, 40]), rnd.choice([1, 3, 8, 17, 64])) for _ in range(6)]
        for align in (1, 8):
            p = make_row_plan(shapes, N, align)
            flats = [random_bits_u32(N, i, r * c).view(np.float32) for i, (r, c) in enumerate(shapes)]
            gathered = np.stack([shard_format(p, r, flats) for r in range(N)])
            for a, b in zip(flats, unshard_format(p, gathered)):
                assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_updates_on_a_row_plan_equal_the_unsharded_update():
    shapes = [(9, 16), (5, 3), (1, 7), (30, 10)]
    numel = [r * c for r, c in shapes]
    N = 4
    p = make_row_plan(shapes, N, 8)
    ws = [normal_f32(2, i, "w", n, 0.02) for i, n in enumerate(numel)]
    gs = [normal_f32(2, i, "g", n, 1e-3) for i, n in enumerate(numel)]
    z = [np.zeros(n, np.float32) for n in numel]
    uw, um, uv, usums = lamb_unsharded_step(ws, gs, z, z, LAMB, 1)
    W = np.stack([shard_format(p, r, ws) for r in range(N)]); G = np.stack([shard_format(p, r, gs) for r in range(N)])
    M = np.zeros_like(W); Vv = np.zeros_like(W); U = np.zeros(W.shape); parts = np.zeros((N, len(shapes), 2))
    for r in range(N):
        M[r], Vv[r], U[r], parts[r] = lamb_shard_partials(p, r, W[r], G[r], M[r], Vv[r], LAMB, 1)
    total = parts.sum(axis=0)
    assert np.allclose(total, usums, rtol=1e-12, atol=0)
    for r in range(N):
        W[r] = lamb_shard_apply(p, W[r], U[r], total, LAMB)
    for a, b in zip(uw, unshard_format(p, W)):
        assert np.max(np.abs(a.astype(np.float64) - b), initial=0.0) <= 4e-9
    # Adam: bit for bit
    A = np.stack([shard_format(p, r, ws) for r in range(N)])
    for r in range(N):
        A[r], _, _ = adam_step(A[r], G[r], np.zeros_like(A[r]), np.zeros_like(A[r]),
                               {"lr": 1e-3, "beta1": 0.9, "beta2": 0.999, "eps": 1e-8}, 1)
    for i, b in enumerate(unshard_format(p, A)):
        a, _, _ = adam_step(ws[i], gs[i], z[i], z[i], {"lr": 1e-3, "beta1": 0.9, "beta2": 0.999, "eps": 1e-8}, 1)
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


# ---------------------------------------------------------------- row / column sums of squares

from oracle import rowcol_sumsq_shard, rowcol_sumsq_unsharded


def test_rowcol_sums_by_loops_and_against_the_norm():
    X = normal_f32(4, 0, "g", 35, 1.0).reshape(5, 7)
    (rows, cols), = rowcol_sumsq_unsharded([X])
    for i in range(5):
        assert abs(rows[i] - sum(float(X[i, j]) ** 2 for j in range(7))) < 1e-12
    for j in range(7):
        assert abs(cols[j] - sum(float(X[i, j]) ** 2 for i in range(5))) < 1e-12
    total = float(np.sum(X.astype(np.float64) ** 2))
    assert abs(rows.sum() - total) < 1e-12 and abs(cols.sum() - total) < 1e-12
    # a transposed operand would swap the two
    (rt, ct), = rowcol_sumsq_unsharded([X.T.copy()])
    assert np.allclose(rt, cols) and np.allclose(ct, rows)


def test_sharded_rowcol_sums_put_together_equal_the_unsharded_ones():
    shapes = [(9, 16), (5, 3), (1, 7), (30, 10), (4, 1), (0, 4)]
    for N in (1, 3, 4, 10):
        p = make_row_plan(shapes, N, 8)
        mats = [normal_f32(6, i, "g", r * c, 1e-2).reshape(r, c) for i, (r, c) in enumerate(shapes)]
        want = rowcol_sumsq_unsharded(mats)
        rows_all = [[] for _ in shapes]
        cols_sum = [np.zeros(c) for _, c in shapes]
        for r in range(N):
            x = shard_format(p, r, [m.ravel() for m in mats])
            # garbage in every padded slot: masks go by position (Section 4.1)
            for i in range(p.V):
                x[p.off[i] + p.real_count(i, r): p.off[i] + p.L[i]] = 9.0
            rs, cp = rowcol_sumsq_shard(p, r, x)
            for i in range(p.V):
                assert rs[i].shape == (p.Lr[i],) and cp[i].shape == (p.cols[i],)
                assert not rs[i][p.real_rows(i, r):].any()                    # padded rows give the identity
                rows_all[i].append(rs[i][:p.real_rows(i, r)])
                cols_sum[i] += cp[i]                                           # the all-reduce over replicas
        for i in range(p.V):
            assert np.allclose(np.concatenate(rows_all[i]), want[i][0], rtol=1e-13, atol=0)   # rows stay sharded
            assert np.allclose(cols_sum[i], want[i][1], rtol=1e-13, atol=0)
