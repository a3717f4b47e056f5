"""GPU parity on the row-granular plan (the paper's own format): formatting bit-exact, updates within tolerance."""
import numpy as np
import pytest
import torch

import oracle
import paper_2004_13336_amd as su
from helpers import (DEV, assert_first_moment_close, assert_second_moment_close, assert_weights_close, f32_hp,
                     pads_are_zero, same_bits, to_dev, to_host)
from workloads import CONFIGS, normal_f32, random_bits_u32

pytestmark = pytest.mark.gpu

LAMB = f32_hp({"lr": 1e-3, "beta1": 0.9, "beta2": 0.999, "eps": 1e-6, "weight_decay": 0.01})
ADAM = f32_hp({"lr": 1e-3, "beta1": 0.9, "beta2": 0.999, "eps": 1e-8, "weight_decay": 0.0})


def _resnet_rows_cols():
    """ResNet-50-shaped variables the way the paper shards them: conv kernels [k,k,Cin,Cout] as (k*k) x (Cin*Cout)
    (leading [3,3] combined, Section 4.1), FC as 2048 x 1000, vectors as n x 1."""
    cfg = [c for c in CONFIGS if c.name == "resnet50"][0]
    out = []
    for s in cfg.shapes:
        if len(s) == 4:
            out.append((s[0] * s[1], s[2] * s[3]))
        elif len(s) == 2:
            out.append((s[0], s[1]))
        else:
            out.append((s[0], 1))
    return out


CASES = [
    ([(9, 16), (5, 3), (1, 7), (0, 4), (12, 10), (3, 0)], 4, 8),      # strides that are not multiples of 8
    ([(9, 65536)], 10, 8),                                            # the paper's example: 9 rows over 10 replicas
    ([(9, 65536), (1000, 1), (64, 1), (7, 4099)], 8, 8),
    ([(33, 100), (2, 5)], 3, 1),
]


@pytest.mark.parametrize("shapes,N,align", CASES)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_row_plan_formatting(shapes, N, align, dtype):
    oplan = oracle.make_row_plan(shapes, N, align)
    plan = su.shard_plan_bind(su.shard_plan_rows([s[0] for s in shapes], [s[1] for s in shapes], N, align))
    assert plan.S == oplan.S
    flats = []
    for i, n in enumerate(oplan.numel):
        bits = random_bits_u32(41, i, n)
        flats.append(bits.view(np.float32) if dtype == "f32" else (bits & 0xFFFF).astype(np.uint16))
    dev_full = [to_dev(f) for f in flats]
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    rows = []
    for r in range(N):
        out = torch.full((max(oplan.S, 1),), 7.0, dtype=tdt, device=DEV)[:oplan.S]
        su.shard_format(plan, r, dev_full, out)
        assert same_bits(to_host(out), oracle.shard_format(oplan, r, flats)), r
        rows.append(out)
    gathered = torch.stack(rows).contiguous()
    if align % 8 == 0:
        allrows = su.gathered_empty(plan, tdt)
        su.shard_format_all(plan, dev_full, allrows)
        assert torch.equal(allrows.contiguous().view(torch.int16 if dtype == "bf16" else torch.int32),
                           gathered.view(torch.int16 if dtype == "bf16" else torch.int32))
    back = [torch.zeros(n, dtype=tdt, device=DEV) for n in oplan.numel]
    su.unshard_format(plan, gathered, back)
    for o, f in zip(back, flats):
        assert same_bits(to_host(o), f)
    plan.free()


def test_row_plan_lamb_and_adam_resnet_shaped():
    shapes = _resnet_rows_cols()
    N = 8
    oplan = oracle.make_row_plan(shapes, N, 8)
    plan = su.shard_plan_bind(su.shard_plan_rows([s[0] for s in shapes], [s[1] for s in shapes], N, 8))
    numel = oplan.numel
    assert sum(numel) == 25557032
    # 3x3 kernels have 9 rows: 2 per replica, so replicas 5..7 hold padding only for them
    ws = [normal_f32(51, i, "w", n, 0.02) for i, n in enumerate(numel)]
    gs = [normal_f32(51, i, "g", n, 1e-3, 1) for i, n in enumerate(numel)]
    z = [np.zeros_like(w) for w in ws]
    uw, um, uv, usums = oracle.lamb_unsharded_step(ws, gs, z, z, LAMB, 1)
    W = to_dev(np.stack([oracle.shard_format(oplan, r, ws) for r in range(N)]))
    G = to_dev(np.stack([oracle.shard_format(oplan, r, gs) for r in range(N)]))
    M = torch.zeros_like(W); V = torch.zeros_like(W)
    nv = len(numel)
    local = torch.zeros((N, ((nv * 2 + 3) // 4) * 4), dtype=torch.float32, device=DEV)     # 16-byte aligned rows
    for r in range(N):
        su.shard_update_lamb_partials(plan, r, W[r], G[r], M[r], V[r], LAMB, 1, local[r])
    total = local[:, :nv * 2].reshape(N, nv, 2).sum(dim=0)
    np.testing.assert_allclose(to_host(total).astype(np.float64), usums, rtol=3e-6, atol=1e-30)
    for r in range(N):
        su.shard_update_lamb_apply(plan, r, W[r], M[r], V[r], LAMB, 1, total)
    Wh = to_host(W)
    for i, (a, b) in enumerate(zip(uw, oracle.unshard_format(oplan, Wh))):
        assert_weights_close(b, a, "var %d" % i)
    for a, b in zip(um, oracle.unshard_format(oplan, to_host(M))):
        assert_first_moment_close(b, a, 1e-3)
    for a, b in zip(uv, oracle.unshard_format(oplan, to_host(V))):
        assert_second_moment_close(b, a)
    for r in range(N):
        assert pads_are_zero(oplan, r, Wh[r])
    # Adam on the same plan
    A = to_dev(np.stack([oracle.shard_format(oplan, r, ws) for r in range(N)]))
    M.zero_(); V.zero_()
    for r in range(N):
        su.shard_update_adam(plan, r, A[r], G[r], M[r], V[r], ADAM, 1)
    for i, b in enumerate(oracle.unshard_format(oplan, to_host(A))):
        a, _, _ = oracle.adam_step(ws[i], gs[i], z[i], z[i], ADAM, 1)
        assert_weights_close(b, a, "adam var %d" % i)
    plan.free()


ROWCOL_CASES = [
    ([(9, 16), (5, 3), (1, 7), (0, 4), (12, 10), (3, 0), (70, 260), (33, 1028), (100, 1)], 4, 8),
    ([(9, 65536)], 10, 8),
    ([(9, 4096), (1000, 1), (64, 1), (7, 4099), (300, 2048)], 8, 8),
    ([(33, 100), (2, 5), (40, 8)], 3, 1),
]


@pytest.mark.parametrize("shapes,N,align", ROWCOL_CASES)
def test_rowcol_sums_of_squares(shapes, N, align):
    oplan = oracle.make_row_plan(shapes, N, align)
    plan = su.shard_plan_bind(su.shard_plan_rows([s[0] for s in shapes], [s[1] for s in shapes], N, align))
    row_off, col_off, total_rows, total_cols = su.shard_plan_rowcol_layout(plan)
    assert total_rows == sum(oplan.Lr) and total_cols == sum(oplan.cols)
    mats = [normal_f32(61, i, "g", n, 1e-2) for i, n in enumerate(oplan.numel)]
    want_full = oracle.rowcol_sumsq_unsharded([m.reshape(s) for m, s in zip(mats, shapes)])
    col_sum = torch.zeros(max(total_cols, 1), dtype=torch.float64, device=DEV)[:total_cols]
    rows_seen = [[] for _ in shapes]
    for r in range(N):
        x = oracle.shard_format(oplan, r, mats)
        for i in range(oplan.V):                                   # garbage in the padding: masked by position
            x[oplan.off[i] + oplan.real_count(i, r): oplan.off[i] + oplan.L[i]] = 9.0
        want_rows, want_cols = oracle.rowcol_sumsq_shard(oplan, r, x)
        row_out = torch.full((total_rows + 4,), -1.0, dtype=torch.float32, device=DEV)
        col_out = torch.full((total_cols + 4,), -1.0, dtype=torch.float32, device=DEV)
        su.shard_reduce_sq_rows_cols(plan, r, to_dev(x), row_out, col_out)
        ro, co = to_host(row_out), to_host(col_out)
        assert (ro[total_rows:] == -1.0).all() and (co[total_cols:] == -1.0).all()
        for i in range(oplan.V):
            np.testing.assert_allclose(ro[row_off[i]:row_off[i] + oplan.Lr[i]].astype(np.float64), want_rows[i],
                                       rtol=3e-6, atol=1e-30)
            np.testing.assert_allclose(co[col_off[i]:col_off[i] + oplan.cols[i]].astype(np.float64), want_cols[i],
                                       rtol=3e-6, atol=1e-30)
            rows_seen[i].append(ro[row_off[i]:row_off[i] + oplan.real_rows(i, r)])
        col_sum += col_out[:total_cols].double()                    # stands in for the all-reduce
        # twice the same bits
        row2 = torch.empty_like(row_out); col2 = torch.empty_like(col_out)
        su.shard_reduce_sq_rows_cols(plan, r, to_dev(x), row2, col2)
        assert torch.equal(row2[:total_rows], row_out[:total_rows]) and torch.equal(col2[:total_cols], col_out[:total_cols])
    cs = col_sum.cpu().numpy()
    for i in range(oplan.V):
        if oplan.cols[i] == 0:                                      # a matrix without columns has no piece at all
            continue
        np.testing.assert_allclose(np.concatenate(rows_seen[i]).astype(np.float64), want_full[i][0], rtol=3e-6, atol=1e-30)
        np.testing.assert_allclose(cs[col_off[i]:col_off[i] + oplan.cols[i]], want_full[i][1], rtol=3e-6, atol=1e-30)
    plan.free()


def test_rowcol_needs_a_row_plan():
    plan = su.shard_plan_bind(su.shard_plan([100, 8], 2))
    with pytest.raises(su.ShardError) as e:
        su.shard_plan_rowcol_layout(plan)
    assert e.value.status == -1
    plan.free()


def test_rowcol_resnet_shaped_full_size():
    shapes = _resnet_rows_cols()
    N = 8
    oplan = oracle.make_row_plan(shapes, N, 8)
    plan = su.shard_plan_bind(su.shard_plan_rows([s[0] for s in shapes], [s[1] for s in shapes], N, 8))
    row_off, col_off, total_rows, total_cols = su.shard_plan_rowcol_layout(plan)
    mats = [normal_f32(62, i, "g", n, 1e-3) for i, n in enumerate(oplan.numel)]
    for r in (0, 4, 7):
        x = oracle.shard_format(oplan, r, mats)
        want_rows, want_cols = oracle.rowcol_sumsq_shard(oplan, r, x)
        row_out = torch.empty(total_rows, dtype=torch.float32, device=DEV)
        col_out = torch.empty(total_cols, dtype=torch.float32, device=DEV)
        su.shard_reduce_sq_rows_cols(plan, r, to_dev(x), row_out, col_out)
        np.testing.assert_allclose(to_host(row_out).astype(np.float64), np.concatenate(want_rows), rtol=3e-6, atol=1e-30)
        np.testing.assert_allclose(to_host(col_out).astype(np.float64), np.concatenate(want_cols), rtol=3e-6, atol=1e-30)
    plan.free()
