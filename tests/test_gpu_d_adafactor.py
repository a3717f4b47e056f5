"""GPU parity of Adafactor on a row plan: every phase against the sharded oracle, the result against
the unsharded oracle, the fused call against the split calls, full-size BERT-shaped variables sampled."""
import numpy as np
import pytest
import torch

import oracle
import paper_2004_13336_amd as su
from helpers import DEV, assert_weights_close, f32_hp, same_bits, to_dev, to_host
from workloads import CONFIGS, normal_f32

pytestmark = pytest.mark.gpu

HP = f32_hp({"eps1": 1e-30, "eps2": 1e-3, "clip_threshold": 1.0, "decay_exponent": 0.8, "max_rho": 1e-2})

CASES = [
    ([(9, 16), (5, 3), (1, 7), (0, 4), (12, 10), (3, 0), (70, 260), (33, 1028), (100, 1)], 4, 8),
    ([(9, 4096), (1000, 1), (64, 1), (7, 4099), (300, 2048)], 8, 8),
    ([(33, 100), (2, 5), (40, 8), (17, 1)], 3, 1),
    ([(64, 1024), (1024, 1)], 1, 8),
]


def _random_case(seed):
    """Seeded random shape list that reaches every tile geometry of the row-plan kernels: pieces of a few
    rows and of hundreds, narrow and very wide matrices, column counts off the 4-element grid, vectors,
    empty variables."""
    rng = np.random.default_rng(4200 + seed)
    shapes = []
    for _ in range(int(rng.integers(2, 7))):
        kind = int(rng.integers(0, 6))
        if kind == 0:
            shapes.append((int(rng.integers(0, 3)), int(rng.integers(0, 5))))
        elif kind == 1:
            shapes.append((int(rng.integers(1, 3000)), 1))                              # vector
        elif kind == 2:
            shapes.append((int(rng.integers(1, 40)), int(rng.integers(1, 6000))))       # few rows, wide
        elif kind == 3:
            shapes.append((int(rng.integers(200, 1500)), int(rng.integers(1, 70))))     # many rows, narrow
        elif kind == 4:
            shapes.append((int(rng.integers(30, 300)), 4 * int(rng.integers(1, 300))))  # aligned columns
        else:
            shapes.append((int(rng.integers(1, 120)), int(rng.integers(250, 1100))))
    return shapes, int(rng.choice([1, 2, 3, 5, 8])), int(rng.choice([1, 4, 8]))


CASES += [_random_case(s) for s in range(6)]


def _split(layout_off, lengths, flat):
    return [flat[o:o + n] for o, n in zip(layout_off, lengths)]


class Rows:
    """[N][S] device rows, each starting on a 16-byte boundary whatever S is."""

    def __init__(self, host_2d, dtype=torch.float32, fill=None):
        N, S = host_2d.shape if fill is None else host_2d
        self.S = S
        pad = -(-max(S, 1) // 8) * 8
        self.buf = torch.zeros((N, pad), dtype=dtype, device=DEV)
        if fill is None:
            self.buf[:, :S] = to_dev(np.ascontiguousarray(host_2d))
        else:
            self.buf.fill_(fill)

    def __getitem__(self, r):
        return self.buf[r][:self.S]

    def host(self):
        return to_host(self.buf[:, :self.S].contiguous())


class Replicas:
    """Device state of all N replicas of one small configuration, plus the oracle's copy."""

    def __init__(self, shapes, N, align, seed):
        self.shapes, self.N = shapes, N
        self.oplan = oracle.make_row_plan(shapes, N, align)
        self.plan = su.shard_plan_bind(su.shard_plan_rows([s[0] for s in shapes], [s[1] for s in shapes], N, align))
        self.row_off, self.col_off, self.total_rows, self.total_cols = su.shard_plan_rowcol_layout(self.plan)
        self.V = len(shapes)
        numel = self.oplan.numel
        self.ws = [normal_f32(seed, i, "w", n, 0.05) for i, n in enumerate(numel)]
        self.W = Rows(np.stack([oracle.shard_format(self.oplan, r, self.ws) for r in range(N)]))
        self.R = torch.zeros((N, max(self.total_rows, 1)), dtype=torch.float32, device=DEV)
        self.C = torch.zeros((N, max(self.total_cols, 1)), dtype=torch.float32, device=DEV)
        # oracle side
        self.o_ws = self.ws
        self.o_R = [np.zeros(s[0], np.float32) for s in shapes]
        self.o_C = [np.zeros(s[1], np.float32) for s in shapes]
        self.seed = seed

    def grads(self, t, scale=1.0):
        gs = [normal_f32(self.seed, i, "g", n, 1e-3 * scale, t) for i, n in enumerate(self.oplan.numel)]
        G = np.stack([oracle.shard_format(self.oplan, r, gs) for r in range(self.N)])
        return gs, G

    def rows_of(self, r, flat):
        return _split(self.row_off, self.oplan.Lr, flat)

    def cols_of(self, flat):
        return _split(self.col_off, self.oplan.cols, flat)


@pytest.mark.parametrize("shapes,N,align", CASES)
def test_every_phase_against_the_sharded_oracle_and_the_result_against_the_unsharded_one(shapes, N, align):
    st = Replicas(shapes, N, align, 61)
    plan, oplan, V = st.plan, st.oplan, st.V
    f = dict(dtype=torch.float32, device=DEV)
    for t in (1, 2):
        gs, G_host = st.grads(t, 20.0 if t == 2 else 1.0)             # the second, larger gradient is clipped
        # padded slots of the gradient hold rubbish: every mask goes by position
        for r in range(N):
            for i in range(V):
                G_host[r][oplan.off[i] + oplan.real_count(i, r):oplan.off[i] + oplan.L[i]] = 7.0
        G = Rows(G_host)
        W_before = st.W.host()
        R_before = to_host(st.R)
        C_before = to_host(st.C)
        # ---- phase 1
        row_sq = torch.full((N, max(st.total_rows, 1)), -1.0, **f)
        col_sq = torch.full((N, max(st.total_cols, 1)), -1.0, **f)
        table = torch.full((N, max(V, 1), 2), -1.0, **f)
        o1 = []
        for r in range(N):
            su.shard_update_adafactor_partials(plan, r, st.W[r], G[r], st.R[r], row_sq[r], col_sq[r], table[r])
            o1.append(oracle.adafactor_shard_partials(oplan, r, W_before[r], G_host[r], st.rows_of(r, R_before[r]), HP))
        row_h, col_h, tab_h = to_host(row_sq), to_host(col_sq), to_host(table)
        for r in range(N):
            for i in range(V):
                rows, cols = shapes[i]
                # the oracle's terms include eps1 (1e-30 per element), far below float32 resolution of g^2 sums
                np.testing.assert_allclose(st.rows_of(r, row_h[r])[i], o1[r][0][i], rtol=3e-6, atol=1e-25)
                np.testing.assert_allclose(st.cols_of(col_h[r])[i], o1[r][1][i], rtol=3e-6, atol=1e-25)
            np.testing.assert_allclose(tab_h[r][:V], o1[r][2], rtol=3e-6, atol=1e-30)
        # ---- the first all-reduce
        col_g, tab_g = col_sq.sum(dim=0), table.sum(dim=0)
        o_col_g = [sum(o1[r][1][i] for r in range(N)) for i in range(V)]
        o_tab_g = sum(o1[r][2] for r in range(N))
        # ---- phase 2
        usq = torch.full((N, max(V, 1)), -1.0, **f)
        o2 = []
        for r in range(N):
            su.shard_update_adafactor_moments(plan, r, G[r], st.R[r], st.C[r], row_sq[r], col_g, tab_g, HP, t, usq[r])
            o2.append(oracle.adafactor_shard_moments(oplan, r, G_host[r], st.rows_of(r, R_before[r]),
                                                     st.cols_of(C_before[r]), o1[r][0], o_col_g, o_tab_g, HP, t))
        R_h, C_h, usq_h = to_host(st.R), to_host(st.C), to_host(usq)
        for r in range(N):
            for i in range(V):
                np.testing.assert_allclose(st.rows_of(r, R_h[r])[i], o2[r][0][i], rtol=4e-6, atol=1e-30)
                real_rows = oplan.real_rows(i, r)
                assert not np.any(st.rows_of(r, R_h[r])[i][real_rows:])          # padded rows keep a zero state
                if shapes[i][1] == 1:
                    assert same_bits(st.cols_of(C_h[r])[i], st.cols_of(C_before[r])[i])   # vectors: C untouched
                else:
                    np.testing.assert_allclose(st.cols_of(C_h[r])[i], o2[r][1][i], rtol=4e-6, atol=1e-30)
            np.testing.assert_allclose(usq_h[r][:V], o2[r][3], rtol=2e-5, atol=1e-30)
            assert same_bits(C_h[r], C_h[0])                                     # every replica holds the same C
        # ---- the second all-reduce, then phase 3 (phase 2 again first: one workspace per plan)
        usq_g = usq.sum(dim=0)
        o_usq_g = sum(o2[r][3] for r in range(N))
        W16 = Rows((N, plan.S), torch.bfloat16, fill=3.0)
        for r in range(N):
            st.R[r].copy_(to_dev(R_before[r])); st.C[r].copy_(to_dev(C_before[r]))
            scratch = torch.empty(max(V, 1), **f)
            su.shard_update_adafactor_moments(plan, r, G[r], st.R[r], st.C[r], row_sq[r], col_g, tab_g, HP, t, scratch)
            su.shard_update_adafactor_apply(plan, r, st.W[r], G[r], tab_g, usq_g, HP, t, w_bf16_out=W16[r])
        assert same_bits(to_host(st.R), R_h) and same_bits(to_host(st.C), C_h)   # phase 2 is reproducible
        W_h = st.W.host()
        W16_h = W16.host()
        for r in range(N):
            want = oracle.adafactor_shard_apply(oplan, r, W_before[r], G_host[r], o2[r][0], o2[r][1], o2[r][2], o_tab_g,
                                                o_usq_g, HP, t)
            assert_weights_close(W_h[r], want, "replica %d step %d" % (r, t))
            # padded slots are untouched, and the bfloat16 copy mirrors all S slots of the GPU's own result
            for i in range(V):
                a, b = oplan.off[i] + oplan.real_count(i, r), oplan.off[i] + oplan.L[i]
                assert same_bits(W_h[r][a:b], W_before[r][a:b])
            assert same_bits(W16_h[r], oracle.f32_to_bf16_bits(W_h[r]))
        # ---- the unsharded definition
        st.o_ws, st.o_R, st.o_C = oracle.adafactor_unsharded_step(shapes, st.o_ws, gs, st.o_R, st.o_C, HP, t)
        full = oracle.unshard_format(oplan, W_h)
        for i in range(V):
            assert_weights_close(full[i], st.o_ws[i], "var %d step %d" % (i, t))
            if shapes[i][0] * shapes[i][1] > 0:
                R_all = np.concatenate([st.rows_of(r, R_h[r])[i] for r in range(N)])[:shapes[i][0]]
                np.testing.assert_allclose(R_all, st.o_R[i], rtol=4e-6)
                if shapes[i][1] > 1:
                    np.testing.assert_allclose(st.cols_of(C_h[0])[i], st.o_C[i], rtol=4e-6)
    plan.free()


def test_fused_call_equals_split_calls_and_is_reproducible():
    shapes, N, r = CASES[1][0], 8, 3
    st = Replicas(shapes, N, 8, 62)
    plan, V = st.plan, st.V
    f = dict(dtype=torch.float32, device=DEV)
    _, G_host = st.grads(1)
    G = Rows(G_host)
    # the other replicas' contributions, from the split calls
    row_sq = torch.zeros((N, st.total_rows), **f); col_sq = torch.zeros((N, st.total_cols), **f)
    table = torch.zeros((N, V, 2), **f); usq = torch.zeros((N, V), **f)
    for q in range(N):
        su.shard_update_adafactor_partials(plan, q, st.W[q], G[q], st.R[q], row_sq[q], col_sq[q], table[q])
    others = [x for x in range(N) if x != r]
    other_col = col_sq[others].sum(dim=0)
    other_tab = table[others].sum(dim=0)
    col_g, tab_g = col_sq[r] + other_col, table[r] + other_tab       # the order the fused call adds in
    R0, C0 = st.R.clone(), st.C.clone()
    for q in range(N):
        su.shard_update_adafactor_moments(plan, q, G[q], st.R[q], st.C[q], row_sq[q], col_g, tab_g, HP, 1, usq[q])
    other_usq = usq[others].sum(dim=0)
    usq_g = usq[r] + other_usq
    W_split = st.W[r].clone()
    Rr, Cr = R0[r].clone(), C0[r].clone()
    su.shard_update_adafactor_moments(plan, r, G[r], Rr, Cr, row_sq[r], col_g, tab_g, HP, 1, torch.empty(V, **f))
    su.shard_update_adafactor_apply(plan, r, W_split, G[r], tab_g, usq_g, HP, 1)
    results = []
    for _ in range(2):
        W_fused, Rf, Cf = st.W[r].clone(), R0[r].clone(), C0[r].clone()
        su.shard_update_adafactor(plan, r, W_fused, G[r], Rf, Cf, HP, 1, other_col_sq=other_col, other_table=other_tab,
                                  other_u_sumsq=other_usq)
        results.append((to_host(W_fused), to_host(Rf), to_host(Cf)))
    assert same_bits(results[0][0], to_host(W_split)) and same_bits(results[0][1], to_host(Rr))
    assert same_bits(results[0][2], to_host(Cr))
    assert all(same_bits(a, b) for a, b in zip(results[0], results[1]))
    assert not same_bits(results[0][0], to_host(st.W[r].clone()))            # it did move the weights
    plan.free()


def _bert_rows_cols():
    """BERT-large-shaped variables as the paper shards them: matrices by rows, vectors as n x 1."""
    cfg = [c for c in CONFIGS if c.name == "bert_large"][0]
    return [(s[0], s[1]) if len(s) == 2 else (s[0], 1) for s in cfg.shapes]


@pytest.mark.parametrize("r", [0, 7])
def test_bert_large_shaped_full_size_sampled_variables(r):
    shapes, N = _bert_rows_cols(), 8
    oplan = oracle.make_row_plan(shapes, N, 8)
    plan = su.shard_plan_bind(su.shard_plan_rows([s[0] for s in shapes], [s[1] for s in shapes], N, 8))
    row_off, col_off, total_rows, total_cols = su.shard_plan_rowcol_layout(plan)
    V = len(shapes)
    assert sum(oplan.numel) == 336226108
    # sampled: the embeddings (type embedding has 2 rows for 8 replicas), a LayerNorm vector, one layer's
    # matrices and biases, the vocabulary bias (ragged rows), the 1024 x 2 head (rows not 16-byte aligned)
    sample = [0, 1, 2, 3, 5, 6, 13, 14, 15, 16, V - 5, V - 3, V - 2, V - 1]
    assert shapes[2] == (2, 1024) and shapes[V - 2] == (1024, 2) and shapes[V - 3] == (30522, 1)
    gen = torch.Generator(device=DEV); gen.manual_seed(77)
    W = torch.empty(plan.S, dtype=torch.float32, device=DEV).normal_(0.0, 0.02, generator=gen)
    G = torch.empty(plan.S, dtype=torch.float32, device=DEV).normal_(0.0, 1e-3, generator=gen)
    R = torch.zeros(total_rows, dtype=torch.float32, device=DEV)
    Cst = torch.zeros(total_cols, dtype=torch.float32, device=DEV)
    other_col = torch.zeros(total_cols, dtype=torch.float32, device=DEV)
    other_tab = torch.zeros((V, 2), dtype=torch.float32, device=DEV)
    other_usq = torch.zeros(V, dtype=torch.float32, device=DEV)
    expect = {}
    for i in sample:
        rows, cols = shapes[i]
        w = normal_f32(71, i, "w", rows * cols, 0.02)
        g = normal_f32(71, i, "g", rows * cols, 1e-3, 1)
        one = oracle.make_row_plan([shapes[i]], N, 8)
        w_sh = [oracle.shard_format(one, q, [w]) for q in range(N)]
        g_sh = [oracle.shard_format(one, q, [g]) for q in range(N)]
        zR = [np.zeros(one.Lr[0], np.float32)]
        p1 = [oracle.adafactor_shard_partials(one, q, w_sh[q], g_sh[q], zR, HP) for q in range(N)]
        col_g = [sum(p1[q][1][0] for q in range(N))]
        tab_g = sum(p1[q][2] for q in range(N))
        p2 = [oracle.adafactor_shard_moments(one, q, g_sh[q], zR, [np.zeros(cols, np.float32)], p1[q][0], col_g, tab_g, HP, 1)
              for q in range(N)]
        usq_g = sum(p2[q][3] for q in range(N))
        (w_ref,), (R_ref,), (C_ref,) = oracle.adafactor_unsharded_step([shapes[i]], [w], [g], [np.zeros(rows, np.float32)],
                                                                      [np.zeros(cols, np.float32)], HP, 1)
        expect[i] = (oracle.shard_format(one, r, [w_ref]), R_ref, C_ref, one)
        seg = slice(oplan.off[i], oplan.off[i] + oplan.L[i])
        W[seg] = to_dev(w_sh[r]); G[seg] = to_dev(g_sh[r])
        # what the other replicas add in the two all-reduces (eps1 terms are far below float32 resolution here)
        if cols > 1:
            other_col[col_off[i]:col_off[i] + cols] = to_dev((col_g[0] - p1[r][1][0]).astype(np.float32))
        other_tab[i] = to_dev((tab_g[0] - p1[r][2][0]).astype(np.float32))
        other_usq[i] = float(usq_g[0] - p2[r][3][0])
    W_before = W.clone()
    su.shard_update_adafactor(plan, r, W, G, R, Cst, HP, 1, other_col_sq=other_col, other_table=other_tab,
                              other_u_sumsq=other_usq)
    W_h, R_h, C_h = to_host(W), to_host(R), to_host(Cst)
    assert np.isfinite(W_h).all()
    for i in sample:
        want, R_ref, C_ref, one = expect[i]
        rows, cols = shapes[i]
        seg = slice(oplan.off[i], oplan.off[i] + oplan.L[i])
        assert_weights_close(W_h[seg], want, "var %d" % i)
        lo = r * one.Lr[0]
        real = one.real_rows(0, r)
        np.testing.assert_allclose(R_h[row_off[i]:row_off[i] + real], R_ref[lo:lo + real], rtol=4e-6)
        if cols > 1:
            np.testing.assert_allclose(C_h[col_off[i]:col_off[i] + cols], C_ref, rtol=4e-6)
    # a relative step: every real element of the sampled variables moved, padding did not
    moved = (W != W_before)
    for i in sample:
        real = oplan.real_count(i, r)
        seg = slice(oplan.off[i], oplan.off[i] + oplan.L[i])
        assert int(moved[seg][:real].sum()) >= int(0.99 * real)
        assert not bool(moved[seg][real:].any())
    plan.free()


def test_argument_errors():
    import ctypes as C
    from paper_2004_13336_amd._lib import AdafactorHP
    flat = su.shard_plan_bind(su.shard_plan([64, 8], 2))
    t = torch.zeros(64, dtype=torch.float32, device=DEV)
    p = C.c_void_p(t.data_ptr())
    hp = AdafactorHP(1e-30, 1e-3, 1.0, 0.8, 1e-2)
    # a flat plan has no rows and columns
    assert su.lib().shard_update_adafactor(flat.handle, 0, p, p, p, p, None, C.byref(hp), 1, None, None, None, None) == -1
    flat.free()
    plan = su.shard_plan_bind(su.shard_plan_rows([16], [8], 2))
    W = torch.zeros(plan.S, dtype=torch.float32, device=DEV)
    R = torch.zeros(8, dtype=torch.float32, device=DEV); Cst = torch.zeros(8, dtype=torch.float32, device=DEV)
    for bad in ({"eps1": 0.0}, {"clip_threshold": 0.0}, {"decay_exponent": 0.0}, {"max_rho": -1.0}, {"eps2": -1.0}):
        with pytest.raises(su.ShardError) as e:
            su.shard_update_adafactor(plan, 0, W, W.clone(), R, Cst, dict(HP, **bad), 1)
        assert e.value.status == -1
    with pytest.raises(su.ShardError):
        su.shard_update_adafactor(plan, 0, W, W.clone(), R, Cst, HP, 0)
    with pytest.raises(su.ShardError):
        su.shard_update_adafactor(plan, 2, W, W.clone(), R, Cst, HP, 1)
    # apply needs the factors of the same replica and step in the workspace
    tab = torch.ones((1, 2), dtype=torch.float32, device=DEV); usq = torch.ones(1, dtype=torch.float32, device=DEV)
    rows_sq = torch.zeros(8, dtype=torch.float32, device=DEV); col_sq = torch.ones(8, dtype=torch.float32, device=DEV)
    with pytest.raises(su.ShardError) as e:
        su.shard_update_adafactor_apply(plan, 0, W, W.clone(), tab, usq, HP, 1)
    assert e.value.status == -5
    su.shard_update_adafactor_moments(plan, 1, W.clone(), R.clone(), Cst.clone(), rows_sq, col_sq, tab, HP, 1, usq.clone())
    with pytest.raises(su.ShardError) as e:
        su.shard_update_adafactor_apply(plan, 0, W, W.clone(), tab, usq, HP, 1)
    assert e.value.status == -5
    with pytest.raises(su.ShardError) as e:
        su.shard_update_adafactor_apply(plan, 1, W, W.clone(), tab, usq, HP, 2)
    assert e.value.status == -5
    su.shard_update_adafactor_apply(plan, 1, W.clone(), W.clone(), tab, usq, HP, 1)
    # zero gradient: eps1 keeps everything finite and the weights stay
    W.normal_(0.0, 0.02)
    before = W.clone()
    su.shard_update_adafactor(plan, 0, W, torch.zeros_like(W), R, Cst, HP, 1)
    assert torch.equal(W, before) and bool(torch.isfinite(R).all()) and bool((R > 0).all())
    plan.free()


def test_late_step_with_a_warm_state():
    # t = 250000: rho = 1/sqrt(t) = 0.002 (below max_rho), beta2 = 1 - t^-0.8 within 5e-5 of 1, and a row/column
    # state that does not come from zero (row and column totals differ, as after loading an old checkpoint)
    shapes, N, t = [(40, 64), (33, 1), (9, 260)], 4, 250000
    st = Replicas(shapes, N, 8, 63)
    plan, oplan, V = st.plan, st.oplan, st.V
    rng = np.random.default_rng(5)
    st.o_R = [rng.uniform(0.5e-6, 2e-6, s[0]).astype(np.float32) * max(s[1], 1) for s in shapes]
    st.o_C = [rng.uniform(0.5e-6, 2e-6, s[1]).astype(np.float32) * s[0] for s in shapes]
    R_host = np.zeros((N, st.total_rows), np.float32)
    C_host = np.zeros(st.total_cols, np.float32)
    for i, (rows, cols) in enumerate(shapes):
        C_host[st.col_off[i]:st.col_off[i] + cols] = st.o_C[i]
        for r in range(N):
            real = oplan.real_rows(i, r)
            R_host[r, st.row_off[i]:st.row_off[i] + real] = st.o_R[i][r * oplan.Lr[i]:r * oplan.Lr[i] + real]
    st.R = to_dev(R_host)
    st.C = to_dev(np.tile(C_host, (N, 1)))
    gs, G_host = st.grads(1)
    G = Rows(G_host)
    f = dict(dtype=torch.float32, device=DEV)
    row_sq = torch.zeros((N, st.total_rows), **f); col_sq = torch.zeros((N, st.total_cols), **f)
    table = torch.zeros((N, V, 2), **f); usq = torch.zeros((N, V), **f)
    for r in range(N):
        su.shard_update_adafactor_partials(plan, r, st.W[r], G[r], st.R[r], row_sq[r], col_sq[r], table[r])
    col_g, tab_g = col_sq.sum(dim=0), table.sum(dim=0)
    R0 = st.R.clone(); C0 = st.C.clone()
    for r in range(N):
        su.shard_update_adafactor_moments(plan, r, G[r], st.R[r], st.C[r], row_sq[r], col_g, tab_g, HP, t, usq[r])
    usq_g = usq.sum(dim=0)
    for r in range(N):
        Rr, Cr = R0[r].clone(), C0[r].clone()
        su.shard_update_adafactor_moments(plan, r, G[r], Rr, Cr, row_sq[r], col_g, tab_g, HP, t, torch.empty(V, **f))
        su.shard_update_adafactor_apply(plan, r, st.W[r], G[r], tab_g, usq_g, HP, t)
    want_w, want_R, want_C = oracle.adafactor_unsharded_step(shapes, st.ws, gs, st.o_R, st.o_C, HP, t)
    full = oracle.unshard_format(oplan, st.W.host())
    R_h, C_h = to_host(st.R), to_host(st.C)
    for i, (rows, cols) in enumerate(shapes):
        assert_weights_close(full[i], want_w[i], "var %d" % i)
        assert np.abs(full[i] - st.ws[i]).max() > 0                   # it moved
        R_all = np.concatenate([st.rows_of(r, R_h[r])[i] for r in range(N)])[:rows]
        np.testing.assert_allclose(R_all, want_R[i], rtol=4e-6)
        if cols > 1:
            np.testing.assert_allclose(st.cols_of(C_h[0])[i], want_C[i], rtol=4e-6)
    plan.free()
