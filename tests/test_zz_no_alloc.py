"""shard_update_lamb_noalloc (the sums of a LAMB step kept in the library's own static device array) against
shard_update_lamb (the same sums in the plan's workspace): same kernels, so the results must agree bit for bit,
and both must meet the oracle's bar.  Two calls in a row, the second on a smaller plan, because every call on a
GPU shares the one array and finds the previous call's contents there."""
import numpy as np
import pytest
import torch

import oracle
import paper_2004_13336_amd as su
from helpers import (DEV, assert_weights_close, f32_hp, gen_weights_grads, shards_of, to_dev, to_host)

pytestmark = pytest.mark.gpu

LAMB = f32_hp({"lr": 1e-3, "beta1": 0.9, "beta2": 0.999, "eps": 1e-6, "weight_decay": 0.01})


def _one_case(numel, N, seed, flags=None):
    """Runs every replica through both entry points; returns nothing, asserts."""
    oplan = oracle.make_plan(numel, N, 8)
    plan_a = su.shard_plan_bind(su.shard_plan(numel, N, 8, flags))
    plan_b = su.shard_plan_bind(su.shard_plan(numel, N, 8, flags))
    nv = len(numel)
    ws, gs = gen_weights_grads(seed, numel, 0.02, 1e-3, 1)
    z = [np.zeros_like(w) for w in ws]
    uw, _, _, usums = oracle.lamb_unsharded_step(ws, gs, z, z, LAMB, 1, flags)
    W0 = to_dev(shards_of(oplan, ws)); G = to_dev(shards_of(oplan, gs))
    # the whole-variable sums, from the existing phase-1 entry point (the all-reduce stand-in)
    local = [torch.zeros((nv, 2), dtype=torch.float32, device=DEV) for _ in range(N)]   # each 16-byte aligned
    for r in range(N):
        su.shard_update_lamb_partials(plan_a, r, W0[r], G[r], torch.zeros_like(W0[r]), torch.zeros_like(W0[r]), LAMB, 1,
                                      local[r])
    total = torch.stack(local).sum(dim=0)
    np.testing.assert_allclose(to_host(total).astype(np.float64), usums, rtol=3e-6, atol=1e-30)
    out = {}
    for name, fn, plan in (("workspace", su.shard_update_lamb, plan_a), ("static", su.shard_update_lamb_noalloc, plan_b)):
        W = W0.clone(); M = torch.zeros_like(W); V = torch.zeros_like(W)
        W16 = torch.zeros(W.shape, dtype=torch.bfloat16, device=DEV)
        mine = [torch.full((nv, 2), -1.0, dtype=torch.float32, device=DEV) for _ in range(N)]
        for r in range(N):
            print("lamb", name, "N=%d r=%d S=%d" % (N, r, oplan.S), flush=True)
            fn(plan, r, W[r], G[r], M[r], V[r], LAMB, 1, other_replicas_sumsq=(total - local[r]).contiguous(),
               local_sumsq_out=mine[r], w_bf16_out=W16[r])
        torch.cuda.synchronize()
        out[name] = (W, M, V, W16, torch.stack(mine))
    for a, b in zip(out["workspace"], out["static"]):
        assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a,
                           b.view(torch.int16) if b.dtype == torch.bfloat16 else b)
    assert torch.equal(out["static"][4], torch.stack(local))
    for i, (a, b) in enumerate(zip(uw, oracle.unshard_format(oplan, to_host(out["static"][0])))):
        assert_weights_close(b, a, "w var %d" % i)
    plan_a.free(); plan_b.free()


def test_lamb_noalloc_matches_lamb_twice_second_smaller():
    big = [70000, 3, 4100, 64, 0, 12345, 2048 * 5 + 17]           # several chunks per variable, ragged tails
    flags = [0, su.SHARD_VAR_NO_DECAY, 0, su.SHARD_VAR_NO_ADAPT, 0, 0, 0]
    _one_case(big, 3, 71, flags)
    small = [515, 9, 2050]                                        # fewer variables, fewer chunks: stale sums lie beyond
    _one_case(small, 2, 72)


def test_lamb_noalloc_refuses_plans_beyond_the_static_limits():
    # more variables than the array has room for: refused on the host, nothing is launched
    V = 32768 + 1
    plan = su.shard_plan_bind(su.shard_plan([8] * V, 1, 8))
    x = torch.zeros(plan.S, dtype=torch.float32, device=DEV)
    with pytest.raises(su.ShardError) as err:
        su.shard_update_lamb_noalloc(plan, 0, x, x.clone(), x.clone(), x.clone(), LAMB, 1)
    assert err.value.status == -6
    plan.free()
