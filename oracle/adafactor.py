"""Adafactor, unsharded and on a row-sharded packed shard (oracle side).  TEST INFRASTRUCTURE ONLY.

The paper names Adafactor, beside LARS, as an optimizer whose weight update contains reduce
operators (Section 3, "Non-elementwise optimizers"; Section 4.1, "Non-elementwise operators"): it
keeps, per matrix, the running row sums and column sums of the squared gradient.  Such reduces
collapse one dimension and pass the other through, so the sharding format may not merge the two;
the row plan (whole rows per replica) keeps them apart.  With rows sharded, the row sums are complete
on the replica that owns the row, the column sums are per-replica partial results that an all-reduce
combines, and padded rows contribute the identity of the sum.

The paper prints no optimizer equations.  The step below is the published definition (Shazeer &
Stern, "Adafactor: Adaptive Learning Rates with Sublinear Memory Cost": the algorithm for matrices
with factored second moments, the one for vectors, update clipping, relative step size, no
momentum), for step t = 1, 2, ...:

    beta2_t = 1 - t^(-decay_exponent)            rho_t = min(max_rho, 1/sqrt(t))
    alpha_t = max(eps2, RMS(X)) * rho_t
    matrix X [n, m]:  R = beta2_t R + (1-beta2_t) * rowsum(G^2 + eps1)        [n]
                      C = beta2_t C + (1-beta2_t) * colsum(G^2 + eps1)        [m]
                      Vhat = R C^T / sum(R)
    vector X [n]:     Vhat = V = beta2_t V + (1-beta2_t) (G^2 + eps1)
    U = G / sqrt(Vhat);   Uhat = U / max(1, RMS(U) / clip_threshold);   X = X - alpha_t * Uhat

A variable of the row plan with cols == 1 is a vector: its row state holds V and it has no column
state.  State arrays (X, R, C) are float32; one step is evaluated in float64 and rounded once.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

import numpy as np

from .plan import Plan

_f64 = np.float64
_f32 = np.float32

DEFAULTS = {"eps1": 1e-30, "eps2": 1e-3, "clip_threshold": 1.0, "decay_exponent": 0.8, "max_rho": 1e-2}


def _hp(hp: Dict[str, float], name: str) -> np.float64:
    return _f64(hp.get(name, DEFAULTS[name]))


def _up(a):
    return np.asarray(a, dtype=_f32).astype(_f64)


def adafactor_schedule(t: int, hp: Dict[str, float]) -> Tuple[np.float64, np.float64]:
    """(beta2_t, rho_t) of step t >= 1."""
    assert t >= 1
    beta2 = _f64(1.0) - _f64(t) ** (-_hp(hp, "decay_exponent"))
    rho = min(_hp(hp, "max_rho"), _f64(1.0) / np.sqrt(_f64(t)))
    return beta2, rho


def adafactor_second_moment(G, R, C, beta2: float, eps1: float):
    """New (R, C, Vhat) of one matrix G [n, m] (float64 in, float64 out).  For m == 1 the variable is
    a vector: R holds the unfactored second moment, C is returned unchanged, Vhat = R[:, None]."""
    G = np.asarray(G, _f64)
    term = G * G + eps1
    if G.shape[1] == 1:
        R = beta2 * R + (1.0 - beta2) * term[:, 0]
        return R, C, R[:, None]
    R = beta2 * R + (1.0 - beta2) * term.sum(axis=1)
    C = beta2 * C + (1.0 - beta2) * term.sum(axis=0)
    return R, C, np.outer(R, C) / R.sum()


def adafactor_unsharded_step(shapes: Sequence[Tuple[int, int]], ws, gs, Rs, Cs, hp: Dict[str, float], t: int):
    """One step on every variable, each a (rows, cols) row-major matrix given flat.  Rs[i] has rows_i
    entries, Cs[i] cols_i entries.  Returns (ws', Rs', Cs') as float32 lists."""
    beta2, rho = adafactor_schedule(t, hp)
    eps1, eps2, d = _hp(hp, "eps1"), _hp(hp, "eps2"), _hp(hp, "clip_threshold")
    out_w, out_R, out_C = [], [], []
    for (rows, cols), w, g, R, C in zip(shapes, ws, gs, Rs, Cs):
        n = rows * cols
        if n == 0:
            out_w.append(np.asarray(w, _f32).copy()); out_R.append(np.asarray(R, _f32).copy())
            out_C.append(np.asarray(C, _f32).copy())
            continue
        X, G = _up(w).reshape(rows, cols), _up(g).reshape(rows, cols)
        R, C, Vhat = adafactor_second_moment(G, _up(R), _up(C), beta2, eps1)
        U = G / np.sqrt(Vhat)
        rms_u = np.sqrt(np.sum(U * U) / n)
        U_hat = U / max(_f64(1.0), rms_u / d)
        alpha = max(eps2, np.sqrt(np.sum(X * X) / n)) * rho
        X = X - alpha * U_hat
        out_w.append(X.reshape(-1).astype(_f32)); out_R.append(R.astype(_f32)); out_C.append(C.astype(_f32))
    return out_w, out_R, out_C


# ---- on a row-sharded packed shard: three local phases around two all-reduces -----------------------

def _piece(plan: Plan, r: int, i: int, x64):
    """(matrix [Lr, cols] of replica r's piece of variable i, mask [Lr] of rows that exist)."""
    Lr, cols = plan.Lr[i], plan.cols[i]
    piece = x64[plan.off[i]:plan.off[i] + Lr * cols].reshape(Lr, cols)
    row_index = r * Lr + np.arange(Lr, dtype=np.int64)          # place in the full matrix: replica offset + index
    return piece, row_index < plan.rows[i]


def adafactor_shard_partials(plan: Plan, r: int, w, g, R_rows: Sequence, hp: Dict[str, float]):
    """Phase 1 (local reduces).  R_rows[i]: replica r's row state of variable i, Lr_i entries.
    Returns (row_terms, col_partials, table): row_terms[i][k] = sum over columns of G^2 + eps1 in row
    k (0 for padded rows); col_partials[i][c] = the same sum over the replica's real rows;
    table[i] = (sum w^2 over real elements, sum of the OLD row state over real rows).  col_partials
    and table are what the first all-reduce adds over replicas."""
    assert plan.rows is not None and 0 <= r < plan.N
    eps1 = _hp(hp, "eps1")
    w64, g64 = _up(w), _up(g)
    row_terms, col_partials = [], []
    table = np.zeros((plan.V, 2), _f64)
    for i in range(plan.V):
        G, real = _piece(plan, r, i, g64)
        X, _ = _piece(plan, r, i, w64)
        term = np.where(real[:, None], G * G + eps1, 0.0)
        row_terms.append(term.sum(axis=1))
        col_partials.append(term.sum(axis=0))
        table[i, 0] = np.sum(np.where(real[:, None], X * X, 0.0))
        table[i, 1] = np.sum(np.where(real, _up(R_rows[i]), 0.0))
    return row_terms, col_partials, table


def adafactor_shard_moments(plan: Plan, r: int, g, R_rows, Cs, row_terms, col_global, table_global,
                            hp: Dict[str, float], t: int):
    """Phase 2.  col_global[i] and table_global are the all-reduced results of phase 1.  Updates the
    row state (local rows) and the column state (the same on every replica), and returns
    (R_rows', Cs', sum_R, u_sumsq): sum_R[i] = the new row state summed over ALL replicas' rows,
    u_sumsq[i] = this replica's sum of U^2 over real elements (for the second all-reduce)."""
    beta2, _ = adafactor_schedule(t, hp)
    g64 = _up(g)
    new_R, new_C = [], []
    sum_R = np.zeros(plan.V, _f64)
    u_sumsq = np.zeros(plan.V, _f64)
    for i in range(plan.V):
        G, real = _piece(plan, r, i, g64)
        R = np.where(real, beta2 * _up(R_rows[i]) + (1.0 - beta2) * np.asarray(row_terms[i], _f64), 0.0)
        vector = plan.cols[i] == 1
        if vector:
            C = _up(Cs[i])
        else:
            C = beta2 * _up(Cs[i]) + (1.0 - beta2) * np.asarray(col_global[i], _f64)
            # sum over all rows of the new row state: the old sum decays, every row gains its term, and
            # the terms of all rows add up to the sum of the all-reduced column terms
            sum_R[i] = beta2 * table_global[i][1] + (1.0 - beta2) * np.sum(np.asarray(col_global[i], _f64))
        if G.size:
            Vhat = R[:, None] if vector else np.outer(R, C) / sum_R[i]
            with np.errstate(divide="ignore", invalid="ignore"):
                U = np.where(real[:, None], G / np.sqrt(Vhat), 0.0)
            u_sumsq[i] = np.sum(U * U)
        new_R.append(R.astype(_f32)); new_C.append(C.astype(_f32))
    return new_R, new_C, sum_R, u_sumsq


def adafactor_shard_apply(plan: Plan, r: int, w, g, R_rows, Cs, sum_R, table_global, u_sumsq_global,
                          hp: Dict[str, float], t: int):
    """Phase 3 with the NEW state and both all-reduced tables; returns w' [S] float32 (padded slots
    are left as they are)."""
    _, rho = adafactor_schedule(t, hp)
    eps2, d = _hp(hp, "eps2"), _hp(hp, "clip_threshold")
    w64, g64 = _up(w), _up(g)
    out = np.asarray(w, _f32).copy()
    for i in range(plan.V):
        n = plan.numel[i]
        if n == 0:
            continue
        G, real = _piece(plan, r, i, g64)
        X, _ = _piece(plan, r, i, w64)
        R, C = _up(R_rows[i]), _up(Cs[i])
        Vhat = R[:, None] if plan.cols[i] == 1 else np.outer(R, C) / sum_R[i]
        with np.errstate(divide="ignore", invalid="ignore"):
            U = G / np.sqrt(Vhat)
        clip = max(_f64(1.0), np.sqrt(u_sumsq_global[i] / n) / d)
        alpha = max(eps2, np.sqrt(table_global[i][0] / n)) * rho
        X = np.where(real[:, None], X - alpha * U / clip, X)
        out[plan.off[i]:plan.off[i] + plan.Lr[i] * plan.cols[i]] = X.reshape(-1).astype(_f32)
    return out
