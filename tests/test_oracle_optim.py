"""Pins for oracle/optim.py: closed forms, library routines, hand cases, the sharding invariant."""
import math

import numpy as np
import pytest
import torch

from oracle import (make_plan, shard_format, unshard_format, adam_step, momentum_step,
                    lamb_unsharded_step, lamb_shard_partials, lamb_shard_apply,
                    VAR_NO_DECAY, VAR_NO_ADAPT)
from workloads import CONFIGS, normal_f32

ADAM = {"lr": 1e-3, "beta1": 0.9, "beta2": 0.999, "eps": 1e-8, "weight_decay": 0.0}
LAMB = {"lr": 1e-3, "beta1": 0.9, "beta2": 0.999, "eps": 1e-6, "weight_decay": 0.01}
F32_HALF_ULP = 2.0 ** -24


def _close(got32, want64, scale=None):
    """got is float64 arithmetic rounded once to float32: within half an ulp (plus float64 noise) of want."""
    want64 = np.asarray(want64, np.float64)
    tol = F32_HALF_ULP * 1.001 * np.maximum(np.abs(want64), 1e-37) + 1e-45
    if scale is not None:
        tol = tol + scale
    assert np.all(np.abs(got32.astype(np.float64) - want64) <= tol), \
        np.max(np.abs(got32.astype(np.float64) - want64) / tol)


def _rand(n, seed, std):
    return normal_f32(seed, 0, "w", n, std)


# ------------------------------------------------------------------------------ Adam

def test_adam_constant_gradient_closed_form():
    # With a constant gradient the bias-corrected moments are exactly g and g^2 at every step,
    # so w_t = w_0 - t * lr * g / (|g| + eps).
    n = 1000
    w0 = _rand(n, 1, 0.02); g = _rand(n, 2, 1e-2)
    w, m, v = w0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    g64 = g.astype(np.float64)
    for t in range(1, 11):
        w, m, v = adam_step(w, g, m, v, ADAM, t)
        if t in (1, 10):
            want = w0.astype(np.float64) - t * ADAM["lr"] * g64 / (np.abs(g64) + ADAM["eps"])
            # state is re-rounded to float32 every step: allow t roundings of w and the moments' rounding
            assert np.max(np.abs(w - want)) <= t * 4e-9
    # first step from zero state, exact up to one rounding
    w1, m1, v1 = adam_step(w0, g, np.zeros(n, np.float32), np.zeros(n, np.float32), ADAM, 1)
    _close(w1, w0.astype(np.float64) - ADAM["lr"] * g64 / (np.abs(g64) + ADAM["eps"]))
    _close(m1, (1.0 - 0.9) * g64)
    _close(v1, (1.0 - 0.999) * g64 * g64)


def test_adam_zero_gradient_leaves_state_alone():
    w = _rand(64, 3, 0.02)
    z = np.zeros(64, np.float32)
    w1, m1, v1 = adam_step(w, z, z, z, ADAM, 1)
    assert np.array_equal(w1, w) and not m1.any() and not v1.any()


@pytest.mark.parametrize("wd", [0.0, 0.01])
def test_adam_matches_torch_float64(wd):
    n = 513
    hp = dict(ADAM, weight_decay=wd)
    w = _rand(n, 4, 0.02); m = np.zeros(n, np.float32); v = np.zeros(n, np.float32)
    p = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([p], lr=hp["lr"], betas=(hp["beta1"], hp["beta2"]), eps=hp["eps"], weight_decay=wd)
    for t in range(1, 6):
        g = normal_f32(40 + t, 0, "g", n, 1e-2)
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        w, m, v = adam_step(w, g, m, v, hp, t)
        # the oracle rounds its state to float32 after every step, torch keeps float64
        assert np.max(np.abs(w - p.detach().numpy())) <= t * 4e-9


# -------------------------------------------------------------------------- momentum

def test_momentum_constant_gradient_closed_form():
    n = 300
    hp = {"lr": 0.1, "mu": 0.9, "weight_decay": 0.0}
    w0 = _rand(n, 5, 0.02); g = _rand(n, 6, 1e-3)
    w, m = w0.copy(), np.zeros(n, np.float32)
    g64 = g.astype(np.float64)
    acc = 0.0
    for k in range(1, 8):
        w, m = momentum_step(w, g, m, hp)
        geo = (1.0 - hp["mu"] ** k) / (1.0 - hp["mu"])
        acc += geo
        assert np.max(np.abs(m - g64 * geo)) <= k * 1e-9
        assert np.max(np.abs(w - (w0 - hp["lr"] * g64 * acc))) <= k * 4e-9


def test_momentum_mu_zero_is_plain_sgd_with_l2():
    n = 100
    hp = {"lr": 0.05, "mu": 0.0, "weight_decay": 5e-5}
    w = _rand(n, 7, 0.02); g = _rand(n, 8, 1e-3)
    w1, m1 = momentum_step(w, g, np.full(n, 9.0, np.float32), hp)
    w64, g64 = w.astype(np.float64), g.astype(np.float64)
    _close(m1, g64 + 5e-5 * w64)
    _close(w1, w64 - 0.05 * (g64 + 5e-5 * w64))


def test_momentum_matches_torch_float64():
    n = 257
    hp = {"lr": 0.1, "mu": 0.9, "weight_decay": 5e-5}
    w = _rand(n, 9, 0.02); m = np.zeros(n, np.float32)
    p = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([p], lr=hp["lr"], momentum=hp["mu"], weight_decay=hp["weight_decay"])
    for t in range(1, 6):
        g = normal_f32(90 + t, 0, "g", n, 1e-3)
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        w, m = momentum_step(w, g, m, hp)
        assert np.max(np.abs(w - p.detach().numpy())) <= t * 4e-9


# ------------------------------------------------------------------------------ LAMB

def _lamb1(w, g, hp, t=1, flags=None, m=None, v=None):
    z = np.zeros_like(w)
    return lamb_unsharded_step([w], [g], [z if m is None else m], [z if v is None else v], hp, t, flags)


def test_lamb_update_norm_equals_lr_times_weight_norm():
    # ||w' - w|| = lr * ratio * ||u|| = lr * ||w||, whatever the gradient is.
    for n, seed in [(1000, 1), (77, 2), (4096, 3)]:
        w = _rand(n, seed, 0.02); g = normal_f32(seed, 1, "g", n, 1e-3)
        (w1,), _, _, _ = _lamb1(w, g, LAMB)
        step = np.linalg.norm(w1.astype(np.float64) - w.astype(np.float64))
        assert abs(step / (LAMB["lr"] * np.linalg.norm(w.astype(np.float64))) - 1.0) < 2e-5


def test_lamb_first_step_without_decay_is_a_scaled_sign_step():
    # t = 1, zero state, wd = 0: u = g / (|g| + eps) ~ sign g, ||u|| ~ sqrt(n), so dw_j = -lr ||w|| / sqrt(n) sign g_j.
    n = 2048
    hp = dict(LAMB, weight_decay=0.0, eps=1e-12)
    w = _rand(n, 11, 0.02); g = normal_f32(11, 1, "g", n, 1e-2)
    (w1,), _, _, sums = _lamb1(w, g, hp)
    wn = np.linalg.norm(w.astype(np.float64))
    want = w.astype(np.float64) - hp["lr"] * wn / math.sqrt(n) * np.sign(g.astype(np.float64))
    assert np.max(np.abs(w1 - want)) < 1e-8
    assert abs(sums[0, 0] - wn * wn) < 1e-12 * wn * wn
    assert abs(sums[0, 1] - n) < 1e-3


def test_lamb_decay_only_closed_form():
    # g = 0 from zero state: u = wd w, ratio = 1/wd, so w' = w (1 - lr) exactly.
    n = 500
    w = _rand(n, 12, 0.02)
    (w1,), (m1,), (v1,), _ = _lamb1(w, np.zeros(n, np.float32), LAMB)
    _close(w1, w.astype(np.float64) * (1.0 - LAMB["lr"]))
    assert not m1.any() and not v1.any()


def test_lamb_single_element_by_hand():
    hp = {"lr": 0.5, "beta1": 0.5, "beta2": 0.75, "eps": 0.0, "weight_decay": 0.25}
    w, g = np.array([2.0], np.float32), np.array([3.0], np.float32)
    # m = 1.5, v = 2.25; m_hat = 3, v_hat = 9; u = 3/3 + 0.25*2 = 1.5; ratio = 2/1.5; w' = 2 - 0.5*(2/1.5)*1.5 = 1
    (w1,), (m1,), (v1,), sums = _lamb1(w, g, hp)
    assert w1[0] == np.float32(1.0) and m1[0] == np.float32(1.5) and v1[0] == np.float32(2.25)
    assert sums[0, 0] == 4.0 and sums[0, 1] == 2.25


def test_lamb_first_step_is_invariant_to_gradient_scale():
    n = 256
    hp = dict(LAMB, eps=0.0)
    w = _rand(n, 13, 0.02); g = normal_f32(13, 1, "g", n, 1e-3)
    (a,), _, _, _ = _lamb1(w, g, hp)
    (b,), _, _, _ = _lamb1(w, g * np.float32(8.0), hp)          # power of two: exact scaling
    assert np.max(np.abs(a.astype(np.float64) - b)) <= 2e-9


@pytest.mark.parametrize("wd", [0.0, 0.01])
def test_lamb_without_adaptation_is_adamw(wd):
    # Trust ratio pinned at 1: w' = w - lr (m_hat / (sqrt v_hat + eps) + wd w), which is AdamW's step.
    n = 400
    hp = dict(LAMB, weight_decay=wd)
    w = _rand(n, 14, 0.02); m = np.zeros(n, np.float32); v = np.zeros(n, np.float32)
    p = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([p], lr=hp["lr"], betas=(hp["beta1"], hp["beta2"]), eps=hp["eps"], weight_decay=wd)
    for t in range(1, 5):
        g = normal_f32(140 + t, 0, "g", n, 1e-3)
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        (w,), (m,), (v,), _ = lamb_unsharded_step([w], [g], [m], [v], hp, t, flags=[VAR_NO_ADAPT])
        assert np.max(np.abs(w - p.detach().numpy())) <= t * 4e-9


def test_lamb_no_decay_flag_drops_only_the_decay_term():
    n = 128
    w = _rand(n, 15, 0.02); g = normal_f32(15, 1, "g", n, 1e-3)
    (a,), _, _, _ = _lamb1(w, g, LAMB, flags=[VAR_NO_DECAY])
    (b,), _, _, _ = _lamb1(w, g, dict(LAMB, weight_decay=0.0))
    assert np.array_equal(a, b)
    (c,), _, _, _ = _lamb1(w, g, LAMB)
    assert not np.array_equal(a, c)


def test_lamb_zero_norm_means_ratio_one():
    n = 16
    z = np.zeros(n, np.float32); g = normal_f32(16, 1, "g", n, 1e-3)
    hp = dict(LAMB, weight_decay=0.0, eps=0.0)
    (w1,), _, _, _ = _lamb1(z, g, hp)                          # ||w|| = 0
    _close(w1, -hp["lr"] * np.sign(g.astype(np.float64)))
    (w2,), _, _, _ = _lamb1(z, z, hp | {"eps": 1e-6})          # both norms 0: nothing moves
    assert not w2.any()


# --------------------------------------------------------- the paper's correctness claim

def _tiny_state(numel, seed, wstd, gstd, step=0):
    ws = [normal_f32(seed, i, "w", n, wstd) for i, n in enumerate(numel)]
    gs = [normal_f32(seed, i, "g", n, gstd, step) for i, n in enumerate(numel)]
    return ws, gs


def _bits_equal(a, b):
    return np.array_equal(a.view(np.uint32), b.view(np.uint32))


@pytest.mark.parametrize("case", ["tiny_config", "ragged"])
def test_sharded_adam_and_momentum_equal_unsharded_bitwise(case):
    """Section 3.1: the update is redundant across replicas, so the N shard updates put back together
    must equal the unsharded update; per element the oracle runs the same arithmetic, so bit for bit."""
    if case == "tiny_config":
        cfg = CONFIGS[0]; numel, N, seed = cfg.numel, 4, cfg.seed
    else:
        numel, N, seed = [0, 1, 5, 6, 7, 64, 1001, 3], 6, 77
    plan = make_plan(numel, N, 8)
    ws, gs = _tiny_state(numel, seed, 0.02, 1e-2)
    zeros = [np.zeros(n, np.float32) for n in numel]
    mom = {"lr": 0.1, "mu": 0.9, "weight_decay": 5e-5}

    # unsharded, 3 steps
    uw, um, uv = [w.copy() for w in ws], [z.copy() for z in zeros], [z.copy() for z in zeros]
    sw, sm = [w.copy() for w in ws], [z.copy() for z in zeros]
    # sharded state
    W = np.stack([shard_format(plan, r, ws) for r in range(N)])
    M = np.zeros_like(W); Vv = np.zeros_like(W)
    W2 = W.copy(); M2 = np.zeros_like(W)
    for t in range(1, 4):
        gs = [normal_f32(seed, i, "g", n, 1e-2, t) for i, n in enumerate(numel)]
        for i in range(len(numel)):
            uw[i], um[i], uv[i] = adam_step(uw[i], gs[i], um[i], uv[i], ADAM, t)
            sw[i], sm[i] = momentum_step(sw[i], gs[i], sm[i], mom)
        for r in range(N):
            G = shard_format(plan, r, gs)
            W[r], M[r], Vv[r] = adam_step(W[r], G, M[r], Vv[r], ADAM, t)
            W2[r], M2[r] = momentum_step(W2[r], G, M2[r], mom)
    for full, shards in ((uw, W), (um, M), (uv, Vv), (sw, W2), (sm, M2)):
        for a, b in zip(full, unshard_format(plan, shards)):
            assert _bits_equal(a, b)
    # padded slots are a fixed point of both updates: still +0.0 bits
    for shards in (W, M, Vv, W2, M2):
        for r in range(N):
            for i in range(plan.V):
                pad = shards[r, plan.off[i] + plan.real_count(i, r): plan.off[i] + plan.L[i]]
                assert not pad.view(np.uint32).any()


@pytest.mark.parametrize("case", ["tiny_config", "ragged"])
def test_sharded_lamb_equals_unsharded(case):
    if case == "tiny_config":
        cfg = CONFIGS[0]; numel, N, seed = cfg.numel, 4, cfg.seed
    else:
        numel, N, seed = [0, 1, 5, 6, 7, 64, 1001, 3], 6, 78
    V = len(numel)
    flags = [0] * V
    flags[2] = VAR_NO_DECAY; flags[-1] = VAR_NO_ADAPT
    plan = make_plan(numel, N, 8)
    ws, _ = _tiny_state(numel, seed, 0.02, 1e-3)
    uw = [w.copy() for w in ws]
    um = [np.zeros(n, np.float32) for n in numel]; uv = [np.zeros(n, np.float32) for n in numel]
    W = np.stack([shard_format(plan, r, ws) for r in range(N)])
    M = np.zeros_like(W); Vv = np.zeros_like(W)
    for t in range(1, 4):
        gs = [normal_f32(seed, i, "g", n, 1e-3, t) for i, n in enumerate(numel)]
        uw, um, uv, usums = lamb_unsharded_step(uw, gs, um, uv, LAMB, t, flags)
        U = np.empty(W.shape, np.float64)
        partials = np.zeros((N, V, 2))
        for r in range(N):
            G = shard_format(plan, r, gs)
            M[r], Vv[r], U[r], partials[r] = lamb_shard_partials(plan, r, W[r], G, M[r], Vv[r], LAMB, t, flags)
        total = partials.sum(axis=0)                       # stands in for the cross-replica all-reduce
        assert np.allclose(total, usums, rtol=1e-12, atol=0)
        for r in range(N):
            W[r] = lamb_shard_apply(plan, W[r], U[r], total, LAMB, flags)
        for a, b in zip(uw, unshard_format(plan, W)):
            assert np.all(np.abs(a.astype(np.float64) - b) <= 1e-6 * (1 + np.abs(a)))
            assert np.max(np.abs(a.astype(np.float64) - b), initial=0.0) <= 4e-9
        for full, shards in ((um, M), (uv, Vv)):
            for a, b in zip(full, unshard_format(plan, shards)):
                assert _bits_equal(a, b)
    for shards in (W, M, Vv):
        for r in range(N):
            for i in range(plan.V):
                pad = shards[r, plan.off[i] + plan.real_count(i, r): plan.off[i] + plan.L[i]]
                assert not pad.view(np.uint32).any()


def test_lamb_partials_mask_padding_by_position_not_by_value():
    # Section 4.1: padded slots must contribute the identity of the reduce, whatever they contain.
    numel = [10, 3]
    N = 4
    plan = make_plan(numel, N, 4)
    ws, gs = _tiny_state(numel, 5, 0.02, 1e-3)
    for r in range(N):
        W = shard_format(plan, r, ws); G = shard_format(plan, r, gs)
        z = np.zeros_like(W)
        _, _, _, clean = lamb_shard_partials(plan, r, W, G, z, z, LAMB, 1)
        Wd, Gd = W.copy(), G.copy()
        for i in range(2):
            real = plan.real_count(i, r)
            Wd[plan.off[i] + real: plan.off[i] + plan.L[i]] = 5.0
            Gd[plan.off[i] + real: plan.off[i] + plan.L[i]] = -3.0
        _, _, _, dirty = lamb_shard_partials(plan, r, Wd, Gd, z, z, LAMB, 1)
        assert np.array_equal(clean, dirty)
        # and the partial over w is the plain sum of squares of the replica's real elements
        for i in range(2):
            piece = ws[i][r * plan.L[i]: r * plan.L[i] + plan.real_count(i, r)].astype(np.float64)
            assert abs(clean[i, 0] - float(np.sum(piece * piece))) <= 1e-15
