"""Pins for oracle/adafactor.py: hand-worked steps, closed forms, the defining property of the
factored estimate, torch's CPU Adafactor as a library cross-check, and sharded == unsharded."""
import math

import numpy as np
import pytest
import torch

from oracle import make_row_plan, shard_format, unshard_format
from oracle.adafactor import (adafactor_schedule, adafactor_second_moment, adafactor_shard_apply,
                              adafactor_shard_moments, adafactor_shard_partials, adafactor_unsharded_step)

HP = {"eps1": 1e-30, "eps2": 1e-3, "clip_threshold": 1.0, "decay_exponent": 0.8, "max_rho": 1e-2}
f32 = np.float32


def _zeros(shapes):
    return [np.zeros(r, f32) for r, _ in shapes], [np.zeros(c, f32) for _, c in shapes]


def test_schedule_values():
    # beta2_t = 1 - t^-0.8, rho_t = min(1e-2, 1/sqrt(t)); worked by hand
    b, rho = adafactor_schedule(1, HP)
    assert b == 0.0 and rho == 1e-2
    b, rho = adafactor_schedule(2, HP)
    assert b == pytest.approx(1.0 - 0.5743491774985175, rel=1e-14) and rho == 1e-2
    b, rho = adafactor_schedule(10 ** 4, HP)
    assert b == pytest.approx(1.0 - 10.0 ** -3.2, rel=1e-14) and rho == pytest.approx(1e-2, rel=1e-15)
    b, rho = adafactor_schedule(10 ** 6, HP)
    assert rho == pytest.approx(1e-3, rel=1e-15)
    assert adafactor_schedule(7, dict(HP, decay_exponent=1.0))[0] == pytest.approx(6.0 / 7.0, rel=1e-15)


def test_two_by_two_matrix_by_hand():
    # G = [[1,2],[3,4]], t = 1 (beta2 = 0): R = [5,25], C = [10,20], sum R = 30,
    # Vhat = [[5/3,10/3],[25/3,50/3]], U^2 = G^2/Vhat = [[0.6,1.2],[1.08,0.96]], mean = 0.96 < 1: no clipping;
    # RMS(X) = sqrt(0.075); alpha = sqrt(0.075) * 0.01
    X = np.array([0.1, -0.2, 0.3, -0.4], f32)
    G = np.array([1.0, 2.0, 3.0, 4.0], f32)
    (w,), (R,), (C,) = adafactor_unsharded_step([(2, 2)], [X], [G], [np.zeros(2, f32)], [np.zeros(2, f32)], HP, 1)
    assert R == pytest.approx([5.0, 25.0], rel=1e-7) and C == pytest.approx([10.0, 20.0], rel=1e-7)
    alpha = math.sqrt(sum(float(x) ** 2 for x in X) / 4) * 0.01
    U = [math.sqrt(0.6), math.sqrt(1.2), math.sqrt(1.08), math.sqrt(0.96)]
    want = [float(x) - alpha * u for x, u in zip(X, U)]
    assert w == pytest.approx(want, abs=2e-8)


def test_vector_by_hand_with_clipping_on_the_second_step():
    # a vector keeps the unfactored second moment.  Step 1: V = g^2, U = sign(g), RMS(U) = 1.
    # Step 2 with a gradient 10x larger: beta2 = 1 - 2^-0.8; V = beta2 g^2 + (1-beta2) 100 g^2; every
    # |U| = 10/sqrt(beta2 + 100 (1-beta2)) = RMS(U) > 1, so Uhat = sign(g) exactly and the step is alpha.
    x0 = np.array([0.5, -0.25, 0.125], f32)
    g = np.array([0.3, -0.2, 0.1], f32)
    shapes = [(3, 1)]
    (x1,), (V1,), (C1,) = adafactor_unsharded_step(shapes, [x0], [g], [np.zeros(3, f32)], [np.zeros(1, f32)], HP, 1)
    a1 = math.sqrt(float(np.sum(x0.astype(np.float64) ** 2)) / 3) * 0.01
    assert x1 == pytest.approx(x0.astype(np.float64) - a1 * np.sign(g), abs=3e-8)      # float32 storage: half an ulp of 0.5
    assert V1 == pytest.approx(g.astype(np.float64) ** 2, rel=1e-7) and C1.tolist() == [0.0]      # no column state
    (x2,), (V2,), _ = adafactor_unsharded_step(shapes, [x1], [10 * g], [V1], [C1], HP, 2)
    b2 = 1.0 - 2.0 ** -0.8
    assert 10.0 / math.sqrt(b2 + 100.0 * (1.0 - b2)) > 1.0
    a2 = math.sqrt(float(np.sum(x1.astype(np.float64) ** 2)) / 3) * 0.01
    assert x2 == pytest.approx(x1.astype(np.float64) - a2 * np.sign(g), abs=3e-8)
    assert V2 == pytest.approx((b2 + 100.0 * (1.0 - b2)) * g.astype(np.float64) ** 2, rel=1e-6)


@pytest.mark.parametrize("d,scale", [(1.0, 1.0), (2.0, 1.0), (0.5, 0.5), (0.25, 0.25)])
def test_rank_one_gradient_first_step_is_a_sign_step(d, scale):
    # G = a b^T: the factored estimate is exact, Vhat = G^2, U = sign(G), RMS(U) = 1;
    # the step is alpha * min(1, d) * sign(G)
    rng = np.random.default_rng(3)
    a, b = rng.uniform(0.5, 2.0, 7) * rng.choice([-1, 1], 7), rng.uniform(0.5, 2.0, 5) * rng.choice([-1, 1], 5)
    G = np.outer(a, b).astype(f32)
    X = rng.normal(0, 0.05, (7, 5)).astype(f32)
    R0, C0 = _zeros([(7, 5)])
    (w,), _, _ = adafactor_unsharded_step([(7, 5)], [X.ravel()], [G.ravel()], R0, C0, dict(HP, clip_threshold=d), 1)
    alpha = math.sqrt(float(np.mean(X.astype(np.float64) ** 2))) * 0.01
    assert w.reshape(7, 5) == pytest.approx(X.astype(np.float64) - alpha * scale * np.sign(G), abs=2e-8)


def test_factored_estimate_keeps_the_row_and_column_sums():
    # the defining property of the factorisation: Vhat has the row sums R and the column sums C
    rng = np.random.default_rng(5)
    G = rng.normal(0, 1, (6, 9))
    R0, C0 = rng.uniform(1, 2, 6), None
    C0 = rng.uniform(1, 2, 9)
    C0 *= R0.sum() / C0.sum()                                     # a consistent state: both sum to the same total
    R, C, Vhat = adafactor_second_moment(G, R0, C0, 0.7, 1e-30)
    brute_R = np.array([0.7 * R0[i] + 0.3 * sum(G[i, j] ** 2 + 1e-30 for j in range(9)) for i in range(6)])
    brute_C = np.array([0.7 * C0[j] + 0.3 * sum(G[i, j] ** 2 + 1e-30 for i in range(6)) for j in range(9)])
    assert R == pytest.approx(brute_R, rel=1e-13) and C == pytest.approx(brute_C, rel=1e-13)
    assert Vhat.sum(axis=1) == pytest.approx(R, rel=1e-12) and Vhat.sum(axis=0) == pytest.approx(C, rel=1e-12)
    for i in range(6):
        for j in range(9):
            assert Vhat[i, j] == pytest.approx(R[i] * C[j] / R.sum(), rel=1e-13)


def test_update_size_and_invariances():
    rng = np.random.default_rng(8)
    shapes = [(12, 8)]
    X = rng.normal(0, 0.05, 96).astype(f32)
    G = rng.normal(0, 1e-3, 96).astype(f32)
    R0, C0 = _zeros(shapes)
    (w,), (R,), (C,) = adafactor_unsharded_step(shapes, [X], [G], R0, C0, HP, 1)
    # gradient scale does not matter (eps1 is far below g^2); a power of two keeps float32 inputs exact
    (w_scaled,), _, _ = adafactor_unsharded_step(shapes, [X], [G * f32(64.0)], R0, C0, HP, 1)
    assert w_scaled == pytest.approx(w, abs=1e-9)
    # relative step size: scaling the weights scales the step (RMS(X) above eps2)
    (w_big,), _, _ = adafactor_unsharded_step(shapes, [X * f32(4.0)], [G], R0, C0, HP, 1)
    assert (w_big.astype(np.float64) - 4.0 * X) == pytest.approx(4.0 * (w.astype(np.float64) - X), abs=1e-8)
    # tiny weights: alpha is floored at eps2 * rho
    Xs = (X * f32(1e-4)).astype(f32)
    (w_small,), _, _ = adafactor_unsharded_step(shapes, [Xs], [G], R0, C0, HP, 1)
    ratio = np.sqrt(np.mean((w_small.astype(np.float64) - Xs) ** 2)) / np.sqrt(np.mean((w.astype(np.float64) - X) ** 2))
    assert ratio == pytest.approx(1e-3 / math.sqrt(float(np.mean(X.astype(np.float64) ** 2))), rel=1e-4)
    # RMS of the step = alpha * min(RMS(U), d), with U rebuilt from the returned state
    U = G.astype(np.float64).reshape(12, 8) / np.sqrt(np.outer(R.astype(np.float64), C.astype(np.float64)) / R.astype(np.float64).sum())
    alpha = math.sqrt(float(np.mean(X.astype(np.float64) ** 2))) * 0.01
    rms_step = math.sqrt(float(np.mean((w.astype(np.float64) - X) ** 2)))
    assert rms_step == pytest.approx(alpha * min(1.0, math.sqrt(float(np.mean(U * U)))), rel=1e-5)
    # zero gradient: eps1 keeps the division defined and the weights stay
    (w0,), (Rz,), _ = adafactor_unsharded_step(shapes, [X], [np.zeros(96, f32)], R0, C0, HP, 1)
    assert np.array_equal(w0, X) and np.all(Rz > 0)


@pytest.mark.parametrize("steps", [1, 5])
def test_against_torch_adafactor_float64(steps):
    # torch's CPU implementation as an independent routine (its eps1 only clamps Vhat from below,
    # which is invisible for non-zero gradients); 2-D parameters are factored, 1-D ones are not
    rng = np.random.default_rng(21)
    shapes = [(9, 6), (5, 1), (4, 16)]
    X = [rng.normal(0, 0.05, r * c).astype(f32) for r, c in shapes]
    params = [torch.tensor(x.astype(np.float64).reshape((r, c) if c > 1 else (r,)), requires_grad=True)
              for x, (r, c) in zip(X, shapes)]
    opt = torch.optim.Adafactor(params, lr=1e-2, beta2_decay=-0.8, eps=(1e-30, 1e-3), d=1.0, weight_decay=0.0,
                                foreach=False)
    Rs, Cs = _zeros(shapes)
    w = X
    for t in range(1, steps + 1):
        G = [(rng.normal(0, 1e-3, r * c) * (3.0 if t == 3 else 1.0)).astype(f32) for r, c in shapes]
        for p, g in zip(params, G):
            p.grad = torch.tensor(g.astype(np.float64).reshape(p.shape))
        opt.step()
        w, Rs, Cs = adafactor_unsharded_step(shapes, w, G, Rs, Cs, HP, t)
        # keep the oracle's float32 rounding of the state out of the comparison: restart torch from the oracle's weights
        for p, wi in zip(params, w):
            assert p.detach().numpy().ravel() == pytest.approx(wi.astype(np.float64), abs=2e-8)
            with torch.no_grad():
                p.copy_(torch.tensor(wi.astype(np.float64).reshape(p.shape)))


CASES = [([(9, 6), (5, 1), (4, 16)], 4), ([(10, 3), (0, 5), (7, 1), (3, 0), (1, 8)], 3), ([(64, 5), (33, 1)], 8),
         ([(3, 4)], 5)]


@pytest.mark.parametrize("shapes,N", CASES)
@pytest.mark.parametrize("align", [1, 8])
def test_sharded_equals_unsharded(shapes, N, align):
    # the paper's correctness claim for a non-elementwise optimizer: N row-sharded updates with the two
    # all-reduces in between, put back together, equal the unsharded update (two steps, state carried)
    rng = np.random.default_rng(N * 100 + align)
    plan = make_row_plan(shapes, N, align)
    X = [rng.normal(0, 0.05, r * c).astype(f32) for r, c in shapes]
    Rs, Cs = _zeros(shapes)
    shard_R = [[np.zeros(plan.Lr[i], f32) for i in range(plan.V)] for _ in range(N)]
    shard_C = [np.zeros(c, f32) for _, c in shapes]
    w_sh = [shard_format(plan, r, X) for r in range(N)]
    w_ref = X
    for t in (1, 2):
        G = [(rng.normal(0, 1e-3, r * c) * (20.0 if t == 2 else 1.0)).astype(f32) for r, c in shapes]
        w_ref, Rs, Cs = adafactor_unsharded_step(shapes, w_ref, G, Rs, Cs, HP, t)
        g_sh = [shard_format(plan, r, G) for r in range(N)]
        garbage = [g.copy() for g in g_sh]
        for r in range(N):                                    # padded slots hold rubbish: masks go by position
            for i in range(plan.V):
                real = plan.real_count(i, r)
                garbage[r][plan.off[i] + real:plan.off[i] + plan.L[i]] = 7.0
        p1 = [adafactor_shard_partials(plan, r, w_sh[r], garbage[r], shard_R[r], HP) for r in range(N)]
        col_global = [sum(p1[r][1][i] for r in range(N)) for i in range(plan.V)]
        table_global = sum(p1[r][2] for r in range(N))
        p2 = [adafactor_shard_moments(plan, r, garbage[r], shard_R[r], shard_C, p1[r][0], col_global, table_global, HP, t)
              for r in range(N)]
        u_global = sum(p2[r][3] for r in range(N))
        for r in range(N):
            assert all(np.array_equal(a, b) for a, b in zip(p2[r][1], p2[0][1]))       # every replica holds the same C
            assert p2[r][2] == pytest.approx(p2[0][2], rel=1e-15)
            w_sh[r] = adafactor_shard_apply(plan, r, w_sh[r], garbage[r], p2[r][0], p2[r][1], p2[r][2], table_global,
                                            u_global, HP, t)
            shard_R[r] = p2[r][0]
        shard_C = p2[0][1]
        full = unshard_format(plan, np.stack(w_sh))
        for i in range(plan.V):
            assert full[i] == pytest.approx(w_ref[i], abs=2e-8)           # one float32 ulp: the float64 sums differ in order
            assert shard_C[i] == pytest.approx(Cs[i], rel=2e-6)
            rows = shapes[i][0]
            if shapes[i][1] == 0:                             # no columns: the piece has no rows either
                continue
            R_all = np.concatenate([shard_R[r][i] for r in range(N)])[:rows]
            assert R_all == pytest.approx(Rs[i], rel=2e-6)
            for r in range(N):                                # padded rows keep a zero state
                assert not np.any(shard_R[r][i][plan.real_rows(i, r):])
        # sum_R of the sharded form equals the plain sum of the unsharded row state
        for i, (rws, cls) in enumerate(shapes):
            if rws * cls > 0 and cls > 1:
                assert p2[0][2][i] == pytest.approx(float(np.sum(Rs[i].astype(np.float64))), rel=1e-6)
