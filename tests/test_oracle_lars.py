"""Pins for the oracle's LARS step (the paper's ResNet-50 optimizer, Section 6, Table 1)."""
import numpy as np
import pytest
import torch

from oracle import (make_plan, shard_format, unshard_format, lars_unsharded_step, lars_shard_partials,
                    lars_shard_apply, VAR_NO_DECAY, VAR_NO_ADAPT)
from workloads import normal_f32

LARS = {"lr": 0.1, "mu": 0.9, "weight_decay": 5e-5, "trust_coeff": 0.001, "eps": 0.0}
HALF_ULP = 2.0 ** -24


def _close(got32, want64):
    want64 = np.asarray(want64, np.float64)
    assert np.all(np.abs(got32.astype(np.float64) - want64) <= HALF_ULP * 1.001 * np.abs(want64) + 1e-45)


def _one(w, g, hp, flags=None, m=None):
    return lars_unsharded_step([w], [g], [np.zeros_like(w) if m is None else m], hp, flags)


def test_first_step_moves_by_lr_times_trust_times_weight_norm():
    # wd = 0, zero momentum: dw = -lr * tc * ||w|| / ||g|| * g, so ||dw|| = lr * tc * ||w||.
    hp = dict(LARS, weight_decay=0.0)
    for n, seed in [(1000, 1), (77, 2)]:
        w = normal_f32(seed, 0, "w", n, 0.02); g = normal_f32(seed, 0, "g", n, 1e-3)
        (w1,), (m1,), sums = _one(w, g, hp)
        w64, g64 = w.astype(np.float64), g.astype(np.float64)
        wn, gn = np.linalg.norm(w64), np.linalg.norm(g64)
        want = w64 - hp["lr"] * hp["trust_coeff"] * wn / gn * g64
        assert np.max(np.abs(w1 - want)) <= 4e-9
        assert abs(sums[0, 0] - wn * wn) <= 1e-12 * wn * wn and abs(sums[0, 1] - gn * gn) <= 1e-12 * gn * gn
        _close(m1, hp["lr"] * hp["trust_coeff"] * wn / gn * g64)


def test_single_element_by_hand():
    hp = {"lr": 0.5, "mu": 0.5, "weight_decay": 0.25, "trust_coeff": 2.0, "eps": 0.0}
    w, g, m = np.array([2.0], np.float32), np.array([3.0], np.float32), np.array([1.0], np.float32)
    # local_lr = 2*2/(3 + 0.25*2) = 8/7; m' = 0.5*1 + 0.5*(8/7)*(3 + 0.5) = 0.5 + 2 = 2.5; w' = 2 - 2.5 = -0.5
    (w1,), (m1,), sums = _one(w, g, hp, m=m)
    assert w1[0] == np.float32(-0.5) and m1[0] == np.float32(2.5)
    assert sums[0, 0] == 4.0 and sums[0, 1] == 9.0


def test_first_step_is_invariant_to_gradient_scale_without_decay():
    hp = dict(LARS, weight_decay=0.0)
    w = normal_f32(3, 0, "w", 256, 0.02); g = normal_f32(3, 0, "g", 256, 1e-3)
    (a,), _, _ = _one(w, g, hp)
    (b,), _, _ = _one(w, g * np.float32(16.0), hp)
    assert np.max(np.abs(a.astype(np.float64) - b)) <= 2e-9


@pytest.mark.parametrize("wd", [0.0, 5e-5])
def test_without_adaptation_is_momentum_sgd(wd):
    # local_lr pinned at 1 and a constant lr: m here equals lr times torch's momentum buffer.
    n = 300
    hp = dict(LARS, weight_decay=wd)
    w = normal_f32(4, 0, "w", n, 0.02); m = np.zeros(n, np.float32)
    p = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([p], lr=hp["lr"], momentum=hp["mu"], weight_decay=wd)
    for t in range(1, 6):
        g = normal_f32(40 + t, 0, "g", n, 1e-3)
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        (w,), (m,), _ = lars_unsharded_step([w], [g], [m], hp, flags=[VAR_NO_ADAPT])
        assert np.max(np.abs(w - p.detach().numpy())) <= t * 4e-9


def test_flags_and_zero_norms():
    n = 64
    w = normal_f32(5, 0, "w", n, 0.02); g = normal_f32(5, 0, "g", n, 1e-3)
    (a,), _, _ = _one(w, g, LARS, flags=[VAR_NO_DECAY])
    (b,), _, _ = _one(w, g, dict(LARS, weight_decay=0.0))
    assert np.array_equal(a, b)
    z = np.zeros(n, np.float32)
    (c,), (mc,), _ = _one(z, g, LARS)                      # ||w|| = 0 -> local_lr = 1: plain SGD step
    _close(c, -LARS["lr"] * g.astype(np.float64))
    (d,), _, _ = _one(w, z, LARS)                          # ||g|| = 0 -> local_lr = 1: w' = w (1 - lr wd)
    _close(d, w.astype(np.float64) * (1.0 - LARS["lr"] * LARS["weight_decay"]))


def test_decay_enters_the_denominator():
    # with g parallel to w the norms are explicit: local_lr = tc ||w|| / (c ||w|| + wd ||w||) = tc / (c + wd)
    n = 50
    w = normal_f32(6, 0, "w", n, 0.02)
    c = np.float32(0.5)
    hp = dict(LARS, weight_decay=0.25, trust_coeff=0.75)
    (w1,), _, _ = _one(w, c * w, hp)
    w64 = w.astype(np.float64)
    _close(w1, w64 - hp["lr"] * (0.75 / (0.5 + 0.25)) * (0.5 + 0.25) * w64)


@pytest.mark.parametrize("numel,N", [([0, 1, 5, 6, 7, 64, 1001, 3], 6), ([128000, 262144, 512], 4)])
def test_sharded_equals_unsharded(numel, N):
    V = len(numel)
    flags = [0] * V
    flags[1] = VAR_NO_ADAPT
    flags[2] = VAR_NO_DECAY
    plan = make_plan(numel, N, 8)
    ws = [normal_f32(7, i, "w", n, 0.02) for i, n in enumerate(numel)]
    uw = [w.copy() for w in ws]; um = [np.zeros(n, np.float32) for n in numel]
    W = np.stack([shard_format(plan, r, ws) for r in range(N)]); M = np.zeros_like(W)
    for t in range(1, 4):
        gs = [normal_f32(7, i, "g", n, 1e-3, t) for i, n in enumerate(numel)]
        uw, um, usums = lars_unsharded_step(uw, gs, um, LARS, flags)
        G = np.stack([shard_format(plan, r, gs) for r in range(N)])
        total = sum(lars_shard_partials(plan, r, W[r], G[r]) for r in range(N))   # the all-reduce
        assert np.allclose(total, usums, rtol=1e-12, atol=0)
        for r in range(N):
            W[r], M[r] = lars_shard_apply(plan, W[r], G[r], M[r], total, LARS, flags)
        for a, b in zip(uw, unshard_format(plan, W)):
            assert np.max(np.abs(a.astype(np.float64) - b), initial=0.0) <= 4e-9
        for a, b in zip(um, unshard_format(plan, M)):
            assert np.max(np.abs(a.astype(np.float64) - b), initial=0.0) <= 1e-11
    for shards in (W, M):                                 # padding is a fixed point
        for r in range(N):
            for i in range(plan.V):
                assert not shards[r, plan.off[i] + plan.real_count(i, r): plan.off[i] + plan.L[i]].view(np.uint32).any()


def test_partials_mask_padding_by_position():
    numel, N = [10, 3], 4
    plan = make_plan(numel, N, 4)
    ws = [normal_f32(8, i, "w", n, 0.02) for i, n in enumerate(numel)]
    gs = [normal_f32(8, i, "g", n, 1e-3) for i, n in enumerate(numel)]
    for r in range(N):
        W = shard_format(plan, r, ws); G = shard_format(plan, r, gs)
        clean = lars_shard_partials(plan, r, W, G)
        for i in range(2):
            real = plan.real_count(i, r)
            W[plan.off[i] + real: plan.off[i] + plan.L[i]] = 5.0
            G[plan.off[i] + real: plan.off[i] + plan.L[i]] = -3.0
        assert np.array_equal(clean, lars_shard_partials(plan, r, W, G))
