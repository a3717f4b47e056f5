"""Optimizer steps, unsharded and on a packed shard (oracle side).

The paper treats the weight update as elementwise operators that read the
gradient, the weight and the auxiliary variables and write the weight and the
auxiliaries back (Section 2.2), plus, for some optimizers, a reduce over the
variable whose padded slots are masked with the identity and whose per-replica
results are combined by an all-reduce (Section 4.1, "Non-elementwise
operators").  The paper prints no optimizer equations; the steps below are the
published definitions:

  Adam      (Kingma & Ba, Algorithm 1; L2 weight decay folded into the gradient)
  momentum  (heavy-ball SGD, no dampening, no Nesterov; L2 decay folded into the gradient)
  LAMB      (You et al., layer-wise adaptive moments: Adam direction plus decoupled
             decay, rescaled per variable by ||w|| / ||direction||)

State arrays are float32; one step is evaluated in float64 and rounded once.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

import numpy as np

from .plan import Plan

VAR_NO_DECAY = 1   # variable is excluded from weight decay
VAR_NO_ADAPT = 2   # variable's trust ratio is fixed at 1

_f64 = np.float64
_f32 = np.float32


def _up(*arrays):
    return tuple(np.asarray(a, dtype=_f32).astype(_f64) for a in arrays)


# --------------------------------------------------------------------------- Adam

def adam_step(w, g, m, v, hp: Dict[str, float], t: int):
    """One Adam step on flat float32 arrays; returns (w', m', v') as float32.  t counts from 1."""
    assert t >= 1
    lr, b1, b2, eps = _f64(hp["lr"]), _f64(hp["beta1"]), _f64(hp["beta2"]), _f64(hp["eps"])
    wd = _f64(hp.get("weight_decay", 0.0))
    w, g, m, v = _up(w, g, m, v)
    if wd != 0.0:
        g = g + wd * w
    m = b1 * m + (1.0 - b1) * g
    v = b2 * v + (1.0 - b2) * g * g
    m_hat = m / (1.0 - b1 ** t)
    v_hat = v / (1.0 - b2 ** t)
    w = w - lr * m_hat / (np.sqrt(v_hat) + eps)
    return w.astype(_f32), m.astype(_f32), v.astype(_f32)


# ----------------------------------------------------------------------- momentum

def momentum_step(w, g, m, hp: Dict[str, float]):
    """One heavy-ball step with L2 weight decay; returns (w', m') as float32."""
    lr, mu = _f64(hp["lr"]), _f64(hp["mu"])
    wd = _f64(hp.get("weight_decay", 0.0))
    w, g, m = _up(w, g, m)
    m = mu * m + (g + wd * w)
    w = w - lr * m
    return w.astype(_f32), m.astype(_f32)


# --------------------------------------------------------------------------- LAMB

def _lamb_direction(w, g, m, v, hp, t: int, decay: bool):
    """Moments and the per-element update direction u (all float64)."""
    b1, b2, eps = _f64(hp["beta1"]), _f64(hp["beta2"]), _f64(hp["eps"])
    wd = _f64(hp.get("weight_decay", 0.0)) if decay else _f64(0.0)
    m = b1 * m + (1.0 - b1) * g
    v = b2 * v + (1.0 - b2) * g * g
    m_hat = m / (1.0 - b1 ** t)
    v_hat = v / (1.0 - b2 ** t)
    u = m_hat / (np.sqrt(v_hat) + eps) + wd * w
    return m, v, u


def _trust_ratio(sum_w2: float, sum_u2: float, adapt: bool) -> float:
    if not adapt:
        return 1.0
    wn, un = np.sqrt(_f64(sum_w2)), np.sqrt(_f64(sum_u2))
    return float(wn / un) if (wn > 0.0 and un > 0.0) else 1.0


def lamb_unsharded_step(ws: Sequence, gs: Sequence, ms: Sequence, vs: Sequence, hp, t: int,
                        flags: Sequence[int] = None):
    """One LAMB step on whole variables (no sharding, no padding).

    Returns (ws', ms', vs', sums) where sums[i] = (sum w^2, sum u^2) of variable i.
    """
    assert t >= 1
    lr = _f64(hp["lr"])
    out_w, out_m, out_v, sums = [], [], [], []
    for i in range(len(ws)):
        fl = 0 if flags is None else int(flags[i])
        w, g, m, v = _up(ws[i], gs[i], ms[i], vs[i])
        m, v, u = _lamb_direction(w, g, m, v, hp, t, decay=not (fl & VAR_NO_DECAY))
        s_w, s_u = float(np.sum(w * w)), float(np.sum(u * u))
        ratio = _trust_ratio(s_w, s_u, adapt=not (fl & VAR_NO_ADAPT))
        w = w - lr * ratio * u
        out_w.append(w.astype(_f32)); out_m.append(m.astype(_f32)); out_v.append(v.astype(_f32))
        sums.append((s_w, s_u))
    return out_w, out_m, out_v, np.array(sums, dtype=_f64).reshape(len(ws), 2)


def lamb_shard_partials(plan: Plan, r: int, w, g, m, v, hp, t: int, flags: Sequence[int] = None):
    """Phase 1 on replica r's packed shard [S].

    Returns (m', v' as float32 [S], u as float64 [S], partial sums float64 [V, 2]).
    The sums run over the slots that hold real elements only: a slot's position
    in the full variable (replica offset + index inside the piece) is compared
    with the variable's length and padded slots contribute 0, whatever they hold.
    """
    assert t >= 1 and 0 <= r < plan.N
    w64, g64, m64, v64 = _up(w, g, m, v)
    m_out = np.empty(plan.S, _f32); v_out = np.empty(plan.S, _f32); u_out = np.empty(plan.S, _f64)
    partial = np.zeros((plan.V, 2), _f64)
    for i in range(plan.V):
        fl = 0 if flags is None else int(flags[i])
        seg = slice(plan.off[i], plan.off[i] + plan.L[i])
        mi, vi, ui = _lamb_direction(w64[seg], g64[seg], m64[seg], v64[seg], hp, t,
                                     decay=not (fl & VAR_NO_DECAY))
        slot = np.arange(plan.L[i], dtype=np.int64)
        position = r * plan.stride[i] + slot            # place in the full variable: replica offset + index
        real = (slot < plan.stride[i]) & (position < plan.numel[i])
        partial[i, 0] = np.sum(np.where(real, w64[seg] * w64[seg], 0.0))
        partial[i, 1] = np.sum(np.where(real, ui * ui, 0.0))
        m_out[seg] = mi.astype(_f32); v_out[seg] = vi.astype(_f32); u_out[seg] = ui
    return m_out, v_out, u_out, partial


def lamb_shard_apply(plan: Plan, w, u, global_sums, hp, flags: Sequence[int] = None):
    """Phase 2: w' = w - lr * ratio_i * u with ratio_i from the all-reduced sums [V, 2]."""
    lr = _f64(hp["lr"])
    (w64,) = _up(w)
    u64 = np.asarray(u, dtype=_f64)
    out = np.empty(plan.S, _f32)
    for i in range(plan.V):
        fl = 0 if flags is None else int(flags[i])
        seg = slice(plan.off[i], plan.off[i] + plan.L[i])
        ratio = _trust_ratio(global_sums[i][0], global_sums[i][1], adapt=not (fl & VAR_NO_ADAPT))
        out[seg] = (w64[seg] - lr * ratio * u64[seg]).astype(_f32)
    return out


# --------------------------------------------------------------------------- LARS
# The paper's ResNet-50 runs use LARS (Section 6, Table 1), its example of an optimizer with a
# reduce over the variable (Section 4.1).  Definition (You, Gitman & Ginsburg): per variable
#     local_lr = trust_coeff * ||w|| / (||g|| + wd * ||w|| + eps)
#     m <- mu * m + lr * local_lr * (g + wd * w) ;   w <- w - m
# with local_lr = 1 when either norm is zero or the variable is flagged VAR_NO_ADAPT.

def _lars_local_lr(sum_w2: float, sum_g2: float, wd: float, hp, adapt: bool) -> float:
    if not adapt:
        return 1.0
    wn, gn = np.sqrt(_f64(sum_w2)), np.sqrt(_f64(sum_g2))
    if not (wn > 0.0 and gn > 0.0):
        return 1.0
    return float(_f64(hp["trust_coeff"]) * wn / (gn + wd * wn + _f64(hp.get("eps", 0.0))))


def _lars_apply(w, g, m, local_lr: float, wd: float, hp):
    lr, mu = _f64(hp["lr"]), _f64(hp["mu"])
    m = mu * m + lr * local_lr * (g + wd * w)
    return w - m, m


def lars_unsharded_step(ws: Sequence, gs: Sequence, ms: Sequence, hp, flags: Sequence[int] = None):
    """One LARS step on whole variables.  Returns (ws', ms', sums) with sums[i] = (sum w^2, sum g^2)."""
    out_w, out_m, sums = [], [], []
    for i in range(len(ws)):
        fl = 0 if flags is None else int(flags[i])
        wd = _f64(0.0) if (fl & VAR_NO_DECAY) else _f64(hp.get("weight_decay", 0.0))
        w, g, m = _up(ws[i], gs[i], ms[i])
        s_w, s_g = float(np.sum(w * w)), float(np.sum(g * g))
        w, m = _lars_apply(w, g, m, _lars_local_lr(s_w, s_g, wd, hp, not (fl & VAR_NO_ADAPT)), wd, hp)
        out_w.append(w.astype(_f32)); out_m.append(m.astype(_f32)); sums.append((s_w, s_g))
    return out_w, out_m, np.array(sums, dtype=_f64).reshape(len(ws), 2)


def lars_shard_partials(plan: Plan, r: int, w, g):
    """Phase 1 on replica r's packed shard: per-variable (sum w^2, sum g^2) over real slots only."""
    assert 0 <= r < plan.N
    w64, g64 = _up(w, g)
    partial = np.zeros((plan.V, 2), _f64)
    for i in range(plan.V):
        seg = slice(plan.off[i], plan.off[i] + plan.L[i])
        slot = np.arange(plan.L[i], dtype=np.int64)
        position = r * plan.stride[i] + slot            # place in the full variable: replica offset + index
        real = (slot < plan.stride[i]) & (position < plan.numel[i])
        partial[i, 0] = np.sum(np.where(real, w64[seg] * w64[seg], 0.0))
        partial[i, 1] = np.sum(np.where(real, g64[seg] * g64[seg], 0.0))
    return partial


def lars_shard_apply(plan: Plan, w, g, m, global_sums, hp, flags: Sequence[int] = None):
    """Phase 2 on a packed shard with the all-reduced sums [V, 2]; returns (w', m') float32 [S]."""
    w64, g64, m64 = _up(w, g, m)
    out_w = np.empty(plan.S, _f32); out_m = np.empty(plan.S, _f32)
    for i in range(plan.V):
        fl = 0 if flags is None else int(flags[i])
        wd = _f64(0.0) if (fl & VAR_NO_DECAY) else _f64(hp.get("weight_decay", 0.0))
        seg = slice(plan.off[i], plan.off[i] + plan.L[i])
        local_lr = _lars_local_lr(global_sums[i][0], global_sums[i][1], wd, hp, not (fl & VAR_NO_ADAPT))
        wi, mi = _lars_apply(w64[seg], g64[seg], m64[seg], local_lr, wd, hp)
        out_w[seg] = wi.astype(_f32); out_m[seg] = mi.astype(_f32)
    return out_w, out_m


# ------------------------------------------------- reductions that keep a dimension (row plan)
# Section 4.1, "Non-elementwise operators": a reduce may collapse some dimensions and pass others
# through; the sharding format must not merge the two kinds, which the row plan guarantees.  With
# rows sharded, a reduce over columns is complete on the replica that owns the row, and a reduce
# over rows yields per-replica partial results that an all-reduce combines; padded rows contribute
# the identity.  The sums of squares below are the two reductions factored second-moment optimizers
# (Adafactor) take of the gradient.

def rowcol_sumsq_unsharded(mats: Sequence):
    """For each 2-D array X: (sum over columns of X^2, one value per row; sum over rows, one per column)."""
    out = []
    for X in mats:
        X64 = np.asarray(X, dtype=_f32).astype(_f64)
        sq = X64 * X64
        out.append((sq.sum(axis=1), sq.sum(axis=0)))
    return out


def rowcol_sumsq_shard(plan: Plan, r: int, x):
    """On replica r's packed shard of a row plan.  Returns (row_sums, col_partials): row_sums[i] has
    Lr_i entries (0 for padded rows), col_partials[i] has cols_i entries summed over the replica's
    real rows only."""
    assert plan.rows is not None and 0 <= r < plan.N
    (x64,) = _up(x)
    row_sums, col_partials = [], []
    for i in range(plan.V):
        Lr, cols = plan.Lr[i], plan.cols[i]
        piece = x64[plan.off[i]:plan.off[i] + Lr * cols].reshape(Lr, cols)
        row_index = r * Lr + np.arange(Lr, dtype=np.int64)          # place in the full matrix
        real = (row_index < plan.rows[i])[:, None]
        sq = np.where(real, piece * piece, 0.0)
        row_sums.append(sq.sum(axis=1))
        col_partials.append(sq.sum(axis=0))
    return row_sums, col_partials
