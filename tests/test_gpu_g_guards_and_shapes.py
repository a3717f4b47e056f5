"""Two things every update kernel must get right whatever its launch shape:
  * it writes inside its outputs only: w, m, v, the bf16 copy, the sums tables, the row/column outputs and the
    Adafactor state sit between canary bands here, on ragged plans with alignments 1, 2 and 8 (the leftover
    elements of the flat kernels, the partly filled tiles of the table-driven ones), and the inputs that are only
    read keep their bits;
  * the launch shapes chosen for large shards (fewer resident workgroups, 128-thread flat kernels, non-temporal
    stores in LAMB's phase 1) compute what the small ones do: element by element against the unsharded oracle
    on shards just past the switch points."""
import numpy as np
import pytest
import torch

import oracle
import paper_2004_13336_amd as su
from helpers import (DEV, Guarded, assert_first_moment_close, assert_second_moment_close, assert_weights_close, f32_hp,
                     gen_weights_grads, same_bits, shards_of, to_dev, to_host)
from workloads import normal_f32

pytestmark = pytest.mark.gpu

ADAM = f32_hp({"lr": 1e-3, "beta1": 0.9, "beta2": 0.999, "eps": 1e-8, "weight_decay": 0.01})
MOM = f32_hp({"lr": 0.1, "mu": 0.9, "weight_decay": 5e-5})
LAMB = f32_hp({"lr": 1e-3, "beta1": 0.9, "beta2": 0.999, "eps": 1e-6, "weight_decay": 0.01})
LARS = f32_hp({"lr": 0.1, "mu": 0.9, "weight_decay": 5e-5, "trust_coeff": 1e-3, "eps": 1e-9})
AF = f32_hp({"eps1": 1e-30, "eps2": 1e-3, "clip_threshold": 1.0, "decay_exponent": 0.8, "max_rho": 1e-2})

RAGGED = [0, 1, 5, 6, 7, 64, 1001, 3, 4096, 4097, 20011, 2048 * 3 + 5]


def _state(oplan, r, ws, gs):
    """Replica r's w, g, m, v (m and v pre-moved so that no lane works on zeros), host side."""
    W = oracle.shard_format(oplan, r, ws)
    G = oracle.shard_format(oplan, r, gs)
    M = oracle.shard_format(oplan, r, [0.1 * g for g in gs])
    V = oracle.shard_format(oplan, r, [(g * g).astype(np.float32) for g in gs])
    return W, G, M, V


@pytest.mark.parametrize("align", [1, 2, 8])
@pytest.mark.parametrize("N", [1, 3])
def test_flat_updates_stay_inside_their_outputs(align, N):
    oplan = oracle.make_plan(RAGGED, N, align)
    plan = su.shard_plan(RAGGED, N, align)
    ws, gs = gen_weights_grads(301, RAGGED, 0.02, 1e-2)
    S = oplan.S
    for r in range(N):
        W, G, M, V = _state(oplan, r, ws, gs)
        print("flat guards align=%d N=%d r=%d S=%d" % (align, N, r, S), flush=True)
        # Adam
        w, g, m, v, w16 = Guarded(S, init=W), Guarded(S, init=G), Guarded(S, init=M), Guarded(S, init=V), Guarded(S, torch.bfloat16)
        su.shard_update_adam(plan, r, w.t, g.t, m.t, v.t, ADAM, 3, w_bf16_out=w16.t)
        torch.cuda.synchronize()
        assert all(x.intact() for x in (w, g, m, v, w16))
        assert same_bits(to_host(g.t), G)
        rw, rm, rv = oracle.adam_step(W, G, M, V, ADAM, 3)
        assert_weights_close(to_host(w.t), rw)
        assert_first_moment_close(to_host(m.t), rm, 1e-2)
        assert_second_moment_close(to_host(v.t), rv)
        assert same_bits(to_host(w16.t), oracle.f32_to_bf16_bits(to_host(w.t)))
        # momentum
        w, g, m, w16 = Guarded(S, init=W), Guarded(S, init=G), Guarded(S, init=M), Guarded(S, torch.bfloat16)
        su.shard_update_momentum(plan, r, w.t, g.t, m.t, MOM, w_bf16_out=w16.t)
        torch.cuda.synchronize()
        assert all(x.intact() for x in (w, g, m, w16))
        assert same_bits(to_host(g.t), G)
        rw, rm = oracle.momentum_step(W, G, M, MOM)
        assert_weights_close(to_host(w.t), rw)
        assert_first_moment_close(to_host(m.t), rm, 1e-2)
        assert same_bits(to_host(w16.t), oracle.f32_to_bf16_bits(to_host(w.t)))
    plan.free()


@pytest.mark.parametrize("align", [1, 2, 8])
@pytest.mark.parametrize("source", ["shard", "full_f32", "full_bf16"])
def test_table_driven_updates_stay_inside_their_outputs(align, source):
    """LAMB and LARS (both phases, fused and split), Adam and momentum from full gradient tensors."""
    N = 3
    flags = [0] * len(RAGGED); flags[5] = su.SHARD_VAR_NO_DECAY; flags[-2] = su.SHARD_VAR_NO_ADAPT
    oplan = oracle.make_plan(RAGGED, N, align)
    plan = su.shard_plan_bind(su.shard_plan(RAGGED, N, align, flags))
    ws, gs = gen_weights_grads(303, RAGGED, 0.02, 1e-2)
    if source == "full_bf16":                   # gradients that bf16 holds exactly, so that both routes see the same values
        gs = [oracle.bf16_bits_to_f32(oracle.f32_to_bf16_bits(g)) for g in gs]
    S, nv = oplan.S, oplan.V
    full_g = None
    if source != "shard":
        full_g = [to_dev(g if source == "full_f32" else oracle.f32_to_bf16_bits(g)) for g in gs]
    for r in range(N):
        W, G, M, V = _state(oplan, r, ws, gs)
        print("table guards align=%d %s r=%d" % (align, source, r), flush=True)
        # ---- LAMB, fused call; the other replicas' sums are zero, so the ratio is this replica's own
        w, g, m, v, w16 = Guarded(S, init=W), Guarded(S, init=G), Guarded(S, init=M), Guarded(S, init=V), Guarded(S, torch.bfloat16)
        local = Guarded(2 * nv)
        if source == "shard":
            su.shard_update_lamb(plan, r, w.t, g.t, m.t, v.t, LAMB, 2, local_sumsq_out=local.t, w_bf16_out=w16.t)
        else:
            su.shard_update_lamb_full_grads(plan, r, w.t, full_g, m.t, v.t, LAMB, 2, local_sumsq_out=local.t, w_bf16_out=w16.t)
        torch.cuda.synchronize()
        assert all(x.intact() for x in (w, g, m, v, w16, local))
        assert same_bits(to_host(g.t), G)
        rm, rv, u, sums = oracle.lamb_shard_partials(oplan, r, W, G, M, V, LAMB, 2, flags)
        np.testing.assert_allclose(to_host(local.t).reshape(nv, 2).astype(np.float64), sums, rtol=3e-6, atol=1e-30)
        rw = oracle.lamb_shard_apply(oplan, W, u, sums, LAMB, flags)
        assert_weights_close(to_host(w.t), rw)
        assert_first_moment_close(to_host(m.t), rm, 1e-2)
        assert_second_moment_close(to_host(v.t), rv)
        assert same_bits(to_host(w16.t), oracle.f32_to_bf16_bits(to_host(w.t)))
        # ---- LARS, split calls
        w, g, m, w16 = Guarded(S, init=W), Guarded(S, init=G), Guarded(S, init=M), Guarded(S, torch.bfloat16)
        local = Guarded(2 * nv)
        if source == "shard":
            su.shard_update_lars_partials(plan, r, w.t, g.t, local.t)
            su.shard_update_lars_apply(plan, r, w.t, g.t, m.t, LARS, local.t, w_bf16_out=w16.t)
        else:
            su.shard_update_lars_partials_full_grads(plan, r, w.t, full_g, local.t)
            su.shard_update_lars_apply_full_grads(plan, r, w.t, full_g, m.t, LARS, local.t, w_bf16_out=w16.t)
        torch.cuda.synchronize()
        assert all(x.intact() for x in (w, g, m, w16, local))
        sums = oracle.lars_shard_partials(oplan, r, W, G)
        np.testing.assert_allclose(to_host(local.t).reshape(nv, 2).astype(np.float64), sums, rtol=3e-6, atol=1e-30)
        rw, rm = oracle.lars_shard_apply(oplan, W, G, M, sums, LARS, flags)
        assert_weights_close(to_host(w.t), rw)
        assert_first_moment_close(to_host(m.t), rm, 1e-2)
        assert same_bits(to_host(w16.t), oracle.f32_to_bf16_bits(to_host(w.t)))
        if source == "shard":
            continue
        # ---- Adam and momentum reading the full gradient tensors
        w, m, v, w16 = Guarded(S, init=W), Guarded(S, init=M), Guarded(S, init=V), Guarded(S, torch.bfloat16)
        su.shard_update_adam_full_grads(plan, r, w.t, full_g, m.t, v.t, ADAM, 3, w_bf16_out=w16.t)
        torch.cuda.synchronize()
        assert all(x.intact() for x in (w, m, v, w16))
        rw, rm, rv = oracle.adam_step(W, G, M, V, ADAM, 3)
        assert_weights_close(to_host(w.t), rw)
        assert_first_moment_close(to_host(m.t), rm, 1e-2)
        assert_second_moment_close(to_host(v.t), rv)
        w, m, w16 = Guarded(S, init=W), Guarded(S, init=M), Guarded(S, torch.bfloat16)
        su.shard_update_momentum_full_grads(plan, r, w.t, full_g, m.t, MOM, w_bf16_out=w16.t)
        torch.cuda.synchronize()
        assert all(x.intact() for x in (w, m, w16))
        rw, rm = oracle.momentum_step(W, G, M, MOM)
        assert_weights_close(to_host(w.t), rw)
        assert_first_moment_close(to_host(m.t), rm, 1e-2)
    plan.free()


@pytest.mark.parametrize("align", [1, 8])
def test_row_plan_reductions_and_adafactor_stay_inside_their_outputs(align):
    """Row/column sums of squares and the three Adafactor phases with every output between canary bands, against the
    sharded oracle."""
    shapes = [(9, 130), (40, 1), (33, 257), (5, 64), (70, 513)]
    N = 4
    rows, cols = [s[0] for s in shapes], [s[1] for s in shapes]
    oplan = oracle.make_row_plan(shapes, N, align)
    plan = su.shard_plan_bind(su.shard_plan_rows(rows, cols, N, align))
    row_off, col_off, total_rows, total_cols = su.shard_plan_rowcol_layout(plan)
    numel = [a * b for a, b in shapes]
    ws, gs = gen_weights_grads(305, numel, 0.02, 1e-2)
    S, nv = oplan.S, oplan.V
    for r in range(N):
        print("row-plan guards align=%d r=%d" % (align, r), flush=True)
        W = oracle.shard_format(oplan, r, ws); G = oracle.shard_format(oplan, r, gs)
        x, ro, co = Guarded(S, init=G), Guarded(total_rows), Guarded(total_cols)
        ro.t.fill_(-1.0); co.t.fill_(-1.0)
        su.shard_reduce_sq_rows_cols(plan, r, x.t, ro.t, co.t)
        torch.cuda.synchronize()
        assert x.intact() and ro.intact() and co.intact() and same_bits(to_host(x.t), G)
        want_rows, want_cols = oracle.rowcol_sumsq_shard(oplan, r, G)
        got_r, got_c = to_host(ro.t), to_host(co.t)
        for i in range(nv):
            np.testing.assert_allclose(got_r[row_off[i]: row_off[i] + len(want_rows[i])], want_rows[i], rtol=4e-6, atol=1e-30)
            np.testing.assert_allclose(got_c[col_off[i]: col_off[i] + len(want_cols[i])], want_cols[i], rtol=4e-6, atol=1e-30)
        # Adafactor, fused call on this replica alone (the other replicas' tables are zero): outputs guarded
        w, g, R, C, w16 = Guarded(S, init=W), Guarded(S, init=G), Guarded(total_rows), Guarded(total_cols), Guarded(S, torch.bfloat16)
        su.shard_update_adafactor(plan, r, w.t, g.t, R.t, C.t, AF, 1, w_bf16_out=w16.t)
        torch.cuda.synchronize()
        assert all(t.intact() for t in (w, g, R, C, w16))
        assert same_bits(to_host(g.t), G)
        assert same_bits(to_host(w16.t), oracle.f32_to_bf16_bits(to_host(w.t)))
        # split calls with guarded intermediate tables give the same bits as the fused call
        w2, R2, C2 = Guarded(S, init=W), Guarded(total_rows), Guarded(total_cols)
        row_sq, col_sq, table, usq = Guarded(total_rows), Guarded(total_cols), Guarded(2 * nv), Guarded(nv)
        su.shard_update_adafactor_partials(plan, r, w2.t, g.t, R2.t, row_sq.t, col_sq.t, table.t)
        su.shard_update_adafactor_moments(plan, r, g.t, R2.t, C2.t, row_sq.t, col_sq.t, table.t, AF, 1, usq.t)
        su.shard_update_adafactor_apply(plan, r, w2.t, g.t, table.t, usq.t, AF, 1)
        torch.cuda.synchronize()
        assert all(t.intact() for t in (w2, R2, C2, row_sq, col_sq, table, usq, g))
        assert torch.equal(w2.t, w.t) and torch.equal(R2.t, R.t) and torch.equal(C2.t, C.t)
    plan.free()


# ---- the launch shapes of large shards ----------------------------------------------------------------

def test_flat_kernels_on_a_shard_past_the_large_switch():
    """2^25 + 7 slots, alignment 1: the 128-thread shape with capped residency, a partly filled last tile and three
    leftover elements; Adam (with the bf16 copy) and momentum against the oracle, outputs guarded."""
    n = (1 << 25) + 7
    oplan = oracle.make_plan([n], 1, 1)
    plan = su.shard_plan([n], 1, 1)
    assert plan.S == n and n % 4 == 3
    ws, gs = gen_weights_grads(307, [n], 0.02, 1e-3)
    W, G = ws[0], gs[0]
    M = (0.1 * G).astype(np.float32); V = (G * G).astype(np.float32)
    print("flat large: adam", flush=True)
    w, g, m, v, w16 = Guarded(n, init=W), Guarded(n, init=G), Guarded(n, init=M), Guarded(n, init=V), Guarded(n, torch.bfloat16)
    su.shard_update_adam(plan, 0, w.t, g.t, m.t, v.t, ADAM, 2, w_bf16_out=w16.t)
    torch.cuda.synchronize()
    assert all(x.intact() for x in (w, g, m, v, w16))
    rw, rm, rv = oracle.adam_step(W, G, M, V, ADAM, 2)
    assert_weights_close(to_host(w.t), rw)
    assert_first_moment_close(to_host(m.t), rm, 1e-3)
    assert_second_moment_close(to_host(v.t), rv)
    assert same_bits(to_host(w16.t), oracle.f32_to_bf16_bits(to_host(w.t)))
    print("flat large: momentum", flush=True)
    w, m = Guarded(n, init=W), Guarded(n, init=M)
    su.shard_update_momentum(plan, 0, w.t, g.t, m.t, MOM)
    torch.cuda.synchronize()
    assert w.intact() and m.intact() and g.intact()
    rw, rm = oracle.momentum_step(W, G, M, MOM)
    assert_weights_close(to_host(w.t), rw)
    assert_first_moment_close(to_host(m.t), rm, 1e-3)
    plan.free()


def test_lamb_and_lars_on_a_shard_past_the_large_switch():
    """One variable of 2^26 + 4099 elements among small ones, one replica: the table-driven kernels run in their
    large-shard shape (LAMB's phase 1 with non-temporal stores, three workgroups per CU); weights, moments and sums
    against the unsharded oracle, element by element."""
    numel = [1000, (1 << 26) + 4099, 70001, 3]
    flags = [0, 0, su.SHARD_VAR_NO_DECAY, su.SHARD_VAR_NO_ADAPT]
    oplan = oracle.make_plan(numel, 1, 8)
    plan = su.shard_plan_bind(su.shard_plan(numel, 1, 8, flags))
    assert plan.S >= 1 << 26
    ws, gs = gen_weights_grads(309, numel, 0.02, 1e-3)
    z = [np.zeros_like(w) for w in ws]
    print("large lamb: oracle", flush=True)
    uw, um, uv, usums = oracle.lamb_unsharded_step(ws, gs, z, z, LAMB, 1, flags)
    W = to_dev(oracle.shard_format(oplan, 0, ws)); G = to_dev(oracle.shard_format(oplan, 0, gs))
    M = torch.zeros_like(W); V = torch.zeros_like(W)
    local = torch.zeros((len(numel), 2), dtype=torch.float32, device=DEV)
    print("large lamb: gpu", flush=True)
    su.shard_update_lamb(plan, 0, W, G, M, V, LAMB, 1, local_sumsq_out=local)
    torch.cuda.synchronize()
    np.testing.assert_allclose(to_host(local).astype(np.float64), usums, rtol=3e-6, atol=1e-30)
    for i, (a, b) in enumerate(zip(uw, oracle.unshard_format(oplan, to_host(W)[None, :]))):
        assert_weights_close(b, a, "lamb w var %d" % i)
    for a, b in zip(um, oracle.unshard_format(oplan, to_host(M)[None, :])):
        assert_first_moment_close(b, a, 1e-3)
    for a, b in zip(uv, oracle.unshard_format(oplan, to_host(V)[None, :])):
        assert_second_moment_close(b, a)
    del uw, um, uv
    print("large lars: oracle", flush=True)
    lw, lm, lsums = oracle.lars_unsharded_step(ws, gs, z, LARS, flags)
    W = to_dev(oracle.shard_format(oplan, 0, ws)); M = torch.zeros_like(W)
    print("large lars: gpu", flush=True)
    su.shard_update_lars(plan, 0, W, G, M, LARS, local_sumsq_out=local)
    torch.cuda.synchronize()
    np.testing.assert_allclose(to_host(local).astype(np.float64), lsums, rtol=3e-6, atol=1e-30)
    for i, (a, b) in enumerate(zip(lw, oracle.unshard_format(oplan, to_host(W)[None, :]))):
        assert_weights_close(b, a, "lars w var %d" % i)
    for a, b in zip(lm, oracle.unshard_format(oplan, to_host(M)[None, :])):
        assert_first_moment_close(b, a, LARS["lr"] * 1e-3, 10)
    plan.free()


def test_every_named_launch_shape_of_adam_gives_the_same_bits():
    """shard_profile_adam_shape runs the update's own kernels in the shape the caller names; whatever the shape, the
    state must come out bit for bit as from shard_update_adam (same arithmetic per element), outputs guarded."""
    n = 3 * 1024 * 1024 + 1027
    plan = su.shard_plan([n], 1, 1)
    ws, gs = gen_weights_grads(311, [n], 0.02, 1e-3)
    W, G = ws[0], gs[0]
    ref = [Guarded(n, init=W), Guarded(n, init=np.zeros(n, np.float32)), Guarded(n, init=np.zeros(n, np.float32))]
    g = Guarded(n, init=G)
    su.shard_update_adam(plan, 0, ref[0].t, g.t, ref[1].t, ref[2].t, ADAM, 1)
    for block in (128, 256):
        for k in (0, 3, 5, 8, 16):
            w, m, v = Guarded(n, init=W), Guarded(n), Guarded(n)
            su.shard_profile_adam_shape(plan, w.t, g.t, m.t, v.t, ADAM, 1, block, k)
            torch.cuda.synchronize()
            assert w.intact() and m.intact() and v.intact() and g.intact(), (block, k)
            assert torch.equal(w.t, ref[0].t) and torch.equal(m.t, ref[1].t) and torch.equal(v.t, ref[2].t), (block, k)
    for block, k in ((64, 0), (256, 2), (128, 17), (256, -1)):
        with pytest.raises(su.ShardError) as err:
            su.shard_profile_adam_shape(plan, ref[0].t, g.t, ref[1].t, ref[2].t, ADAM, 1, block, k)
        assert err.value.status == -1
    plan.free()
