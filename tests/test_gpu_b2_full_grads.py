"""GPU parity of the updates that read the gradient in place from the full tensors (formatting fused
into the update, Section 5.1): bit for bit what shard_format followed by the plain update gives, and
within the usual bounds of the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2004_13336_amd as su
from helpers import DEV, assert_weights_close, f32_hp, pads_are_zero, shards_of, to_dev, to_host
from workloads import CONFIGS, normal_f32

pytestmark = pytest.mark.gpu

ADAM = f32_hp({"lr": 1e-3, "beta1": 0.9, "beta2": 0.999, "eps": 1e-8, "weight_decay": 0.01})
MOM = f32_hp({"lr": 0.1, "mu": 0.9, "weight_decay": 5e-5})
LAMB = f32_hp({"lr": 1e-3, "beta1": 0.9, "beta2": 0.999, "eps": 1e-6, "weight_decay": 0.01})
LARS = f32_hp({"lr": 0.1, "mu": 0.9, "weight_decay": 5e-5, "trust_coeff": 0.001, "eps": 0.0})

RAGGED = [0, 1, 5, 6, 7, 64, 1001, 3, 4096, 4097, 20011, 2048, 8191]


def _cfg(name):
    return [c for c in CONFIGS if c.name == name][0]


def _bits_equal(a, b):
    return a.dtype == b.dtype and a.shape == b.shape and torch.equal(a.view(torch.int16 if a.element_size() == 2 else torch.int32),
                                                                     b.view(torch.int16 if b.element_size() == 2 else torch.int32))


def _aligned(n, dtype=torch.float32, fill=None):
    """A length-n device vector that starts on a 16-byte boundary whatever n is."""
    t = torch.empty((n + 7) // 8 * 8 + 8, dtype=dtype, device=DEV)
    t = t[:n]
    if fill is not None:
        t.fill_(fill)
    return t


def _full_grads(numel, seed, step, dtype, misalign):
    """Full gradient tensors carved from one buffer; with misalign every tensor starts one element past a
    16-byte boundary (float32) or at an odd element (bfloat16)."""
    gap = 1 if misalign else 0
    starts, pos = [], gap
    for n in numel:
        starts.append(pos)
        pos += (n + 7) // 8 * 8 + gap * 8
    buf = torch.zeros(pos + 8, dtype=dtype, device=DEV)
    out = []
    for i, n in enumerate(numel):
        if not misalign:
            assert starts[i] % 8 == 0
        view = buf[starts[i]: starts[i] + n]
        view.copy_(torch.from_numpy(normal_f32(seed, i, "g", n, 1e-3, step)).to(DEV).to(dtype))
        out.append(view)
    return out


class _State:
    """Replica r's shard state, twice: one copy per route."""

    def __init__(self, plan, oplan, r, seed, numel, n_streams):
        ws = [normal_f32(seed, i, "w", n, 0.02) for i, n in enumerate(numel)]
        w0 = to_dev(oracle.shard_format(oplan, r, ws))
        self.S = plan.S
        self.routes = []
        for _ in range(2):
            w = _aligned(self.S); w.copy_(w0)
            st = [w] + [_aligned(self.S, fill=0.0) for _ in range(n_streams - 1)]
            self.routes.append((st, _aligned(self.S, torch.bfloat16, fill=0.0)))
        self.g = _aligned(self.S)

    def same(self):
        (a, a16), (b, b16) = self.routes
        return all(_bits_equal(x, y) for x, y in zip(a, b)) and _bits_equal(a16, b16)


def _sums(nv):
    return _aligned(2 * nv, fill=-1.0)


@pytest.mark.parametrize("misalign", [False, True])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("align", [8, 4, 1])
def test_every_update_from_full_gradients_equals_format_then_update(align, dtype, misalign):
    numel, N, seed = RAGGED, 6, 321
    print("full grads", align, dtype, misalign, flush=True)
    oplan = oracle.make_plan(numel, N, align)
    nv = len(numel)
    flags = [0] * nv; flags[2] = su.SHARD_VAR_NO_DECAY; flags[-1] = su.SHARD_VAR_NO_ADAPT
    plan = su.shard_plan_bind(su.shard_plan(numel, N, align, flags))
    for r in range(N):
        adam = _State(plan, oplan, r, seed, numel, 3)
        mom = _State(plan, oplan, r, seed, numel, 2)
        lamb = _State(plan, oplan, r, seed, numel, 3)
        lamb_split = _State(plan, oplan, r, seed, numel, 3)
        lars = _State(plan, oplan, r, seed, numel, 2)
        lars_split = _State(plan, oplan, r, seed, numel, 2)
        for t in (1, 2):
            full = _full_grads(numel, seed, t, dtype, misalign)
            g = adam.g
            su.shard_format(plan, r, full, g)                     # float32 shard gradient, padding +0.0
            # Adam
            (a, a16), (b, b16) = adam.routes
            su.shard_update_adam(plan, r, a[0], g, a[1], a[2], ADAM, t, w_bf16_out=a16)
            su.shard_update_adam_full_grads(plan, r, b[0], full, b[1], b[2], ADAM, t, w_bf16_out=b16)
            assert adam.same(), "adam r=%d t=%d" % (r, t)
            # momentum
            (a, a16), (b, b16) = mom.routes
            su.shard_update_momentum(plan, r, a[0], g, a[1], MOM, w_bf16_out=a16)
            su.shard_update_momentum_full_grads(plan, r, b[0], full, b[1], MOM, w_bf16_out=b16)
            assert mom.same(), "momentum r=%d t=%d" % (r, t)
            # LAMB, one call
            other = _sums(nv); other.copy_(torch.rand(2 * nv, device=DEV) * 1e-3)
            la, lb = _sums(nv), _sums(nv)
            (a, a16), (b, b16) = lamb.routes
            su.shard_update_lamb(plan, r, a[0], g, a[1], a[2], LAMB, t, other_replicas_sumsq=other, local_sumsq_out=la,
                                 w_bf16_out=a16)
            su.shard_update_lamb_full_grads(plan, r, b[0], full, b[1], b[2], LAMB, t, other_replicas_sumsq=other,
                                            local_sumsq_out=lb, w_bf16_out=b16)
            assert lamb.same() and _bits_equal(la, lb), "lamb r=%d t=%d" % (r, t)
            # LAMB, phase by phase
            (a, a16), (b, b16) = lamb_split.routes
            su.shard_update_lamb_partials(plan, r, a[0], g, a[1], a[2], LAMB, t, la)
            su.shard_update_lamb_partials_full_grads(plan, r, b[0], full, b[1], b[2], LAMB, t, lb)
            assert _bits_equal(la, lb)
            tot = _sums(nv); tot.copy_(la + other)
            su.shard_update_lamb_apply(plan, r, a[0], a[1], a[2], LAMB, t, tot, w_bf16_out=a16)
            su.shard_update_lamb_apply(plan, r, b[0], b[1], b[2], LAMB, t, tot, w_bf16_out=b16)
            assert lamb_split.same(), "lamb split r=%d t=%d" % (r, t)
            # LARS, one call and phase by phase
            (a, a16), (b, b16) = lars.routes
            su.shard_update_lars(plan, r, a[0], g, a[1], LARS, other_replicas_sumsq=other, local_sumsq_out=la,
                                 w_bf16_out=a16)
            su.shard_update_lars_full_grads(plan, r, b[0], full, b[1], LARS, other_replicas_sumsq=other,
                                            local_sumsq_out=lb, w_bf16_out=b16)
            assert lars.same() and _bits_equal(la, lb), "lars r=%d t=%d" % (r, t)
            (a, a16), (b, b16) = lars_split.routes
            su.shard_update_lars_partials(plan, r, a[0], g, la)
            su.shard_update_lars_partials_full_grads(plan, r, b[0], full, lb)
            assert _bits_equal(la, lb)
            tot.copy_(la + other)
            su.shard_update_lars_apply(plan, r, a[0], g, a[1], LARS, tot, w_bf16_out=a16)
            su.shard_update_lars_apply_full_grads(plan, r, b[0], full, b[1], LARS, tot, w_bf16_out=b16)
            assert lars_split.same(), "lars split r=%d t=%d" % (r, t)
        # padding untouched by every route
        for st in (adam, mom, lamb, lars):
            for t_ in st.routes[1][0]:
                assert pads_are_zero(oplan, r, to_host(t_))
    plan.free()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_adam_and_lamb_from_full_gradients_against_the_unsharded_oracle(dtype):
    """Independent of the formatting kernels: all replicas updated from the full tensors, put back
    together by the oracle and compared with the oracle's unsharded step on the same (rounded) gradients."""
    numel, N, align, seed = RAGGED, 5, 8, 77
    nv = len(numel)
    oplan = oracle.make_plan(numel, N, align)
    plan = su.shard_plan_bind(su.shard_plan(numel, N, align))
    ws = [normal_f32(seed, i, "w", n, 0.02) for i, n in enumerate(numel)]
    W0 = shards_of(oplan, ws)
    for which in ("adam", "lamb"):
        uw = [w.copy() for w in ws]; um = [np.zeros_like(w) for w in ws]; uv = [np.zeros_like(w) for w in ws]
        W = [to_dev(W0[r]) for r in range(N)]
        M = [torch.zeros_like(w) for w in W]; V = [torch.zeros_like(w) for w in W]
        for t in (1, 2, 3):
            full = _full_grads(numel, seed, t, dtype, False)
            gs = [to_host(f.to(torch.float32)) for f in full]                 # what the kernels see
            if which == "adam":
                for i in range(nv):
                    uw[i], um[i], uv[i] = oracle.adam_step(uw[i], gs[i], um[i], uv[i], ADAM, t)
                for r in range(N):
                    su.shard_update_adam_full_grads(plan, r, W[r], full, M[r], V[r], ADAM, t)
            else:
                uw, um, uv, usums = oracle.lamb_unsharded_step(uw, gs, um, uv, LAMB, t, None)
                local = torch.zeros((N, (2 * nv + 3) // 4 * 4), device=DEV)
                for r in range(N):
                    su.shard_update_lamb_partials_full_grads(plan, r, W[r], full, M[r], V[r], LAMB, t, local[r])
                total = local[:, :2 * nv].sum(dim=0).contiguous()
                np.testing.assert_allclose(to_host(total).astype(np.float64).reshape(nv, 2), usums, rtol=3e-6, atol=1e-30)
                for r in range(N):
                    su.shard_update_lamb_apply(plan, r, W[r], M[r], V[r], LAMB, t, total)
            Wh = np.stack([to_host(w) for w in W])
            for i, (a, b) in enumerate(zip(uw, oracle.unshard_format(oplan, Wh))):
                assert_weights_close(b, a, "%s w var %d t=%d" % (which, i, t))
            for r in range(N):
                assert pads_are_zero(oplan, r, Wh[r])
    plan.free()


def test_row_plan_pieces_from_full_gradients():
    """On a row plan the pieces sit Lr*cols apart in the full tensor (not L) and need not be 16-byte aligned."""
    rows, cols, N = [9, 7, 130, 1, 64], [33, 1, 5, 1000, 64], 4
    oplan = oracle.make_row_plan(list(zip(rows, cols)), N, 8)
    plan = su.shard_plan_bind(su.shard_plan_rows(rows, cols, N, 8))
    numel = [a * b for a, b in zip(rows, cols)]
    nv = len(numel)
    for r in range(N):
        st = _State(plan, oplan, r, 55, numel, 3)
        full = _full_grads(numel, 55, 1, torch.float32, False)
        su.shard_format(plan, r, full, st.g)
        la, lb = _sums(nv), _sums(nv)
        (a, a16), (b, b16) = st.routes
        su.shard_update_lamb(plan, r, a[0], st.g, a[1], a[2], LAMB, 1, local_sumsq_out=la, w_bf16_out=a16)
        su.shard_update_lamb_full_grads(plan, r, b[0], full, b[1], b[2], LAMB, 1, local_sumsq_out=lb, w_bf16_out=b16)
        assert st.same() and _bits_equal(la, lb), r
    plan.free()


@pytest.mark.parametrize("case", ["bert_large_N8", "resnet50_N32"])
def test_full_size_from_full_gradients(case):
    """The launch configuration the bench times (BERT-shaped, N = 8), and the ResNet-shaped list at 32
    replicas, where the last replica holds all-padding pieces."""
    name, N = ("bert_large", 8) if case.startswith("bert") else ("resnet50", 32)
    cfg = _cfg(name)
    plan = su.shard_plan_bind(su.shard_plan(cfg.numel, N, 8))
    S, nv = plan.S, len(cfg.numel)
    flat = torch.empty(cfg.total, device=DEV).normal_(0.0, cfg.grad_std)
    full, pos = [], 0
    for n in cfg.numel:
        full.append(flat[pos:pos + n]); pos += n
    full = su.FullTensors(plan, full)
    for r in (0, N - 1):
        print(case, "r", r, flush=True)
        g = torch.empty(S, device=DEV)
        su.shard_format(plan, r, full, g)
        w0 = torch.empty(S, device=DEV).normal_(0.0, 0.02)
        outs = []
        for route in (0, 1):
            w = w0.clone(); m = torch.zeros_like(w); v = torch.zeros_like(w); loc = _sums(nv)
            m2 = torch.zeros_like(w); w2 = w0.clone()
            for t in (1, 2):
                if route == 0:
                    su.shard_update_lamb(plan, r, w, g, m, v, LAMB, t, local_sumsq_out=loc)
                    su.shard_update_lars(plan, r, w2, g, m2, LARS)
                else:
                    su.shard_update_lamb_full_grads(plan, r, w, full, m, v, LAMB, t, local_sumsq_out=loc)
                    su.shard_update_lars_full_grads(plan, r, w2, full, m2, LARS)
            outs.append((w, m, v, loc, w2, m2))
        for a, b in zip(*outs):
            assert _bits_equal(a, b)
        del outs, g, w0
    plan.free()


def test_argument_errors():
    numel, N = [64, 5, 0], 2
    plan = su.shard_plan_bind(su.shard_plan(numel, N, 8))
    S = plan.S
    w, m, v = (_aligned(S, fill=0.0) for _ in range(3))
    full = [torch.zeros(n, device=DEV) for n in numel]
    loc = _sums(3)
    su.shard_update_adam_full_grads(plan, 0, w, full, m, v, ADAM, 1)                       # fine, the empty variable included
    with pytest.raises(ValueError):
        su.shard_update_adam_full_grads(plan, 0, w, full[:2], m, v, ADAM, 1)               # binding: wrong count
    with pytest.raises(ValueError):
        su.shard_update_lamb_full_grads(plan, 0, w, [full[0], full[1].double(), full[2]], m, v, LAMB, 1)
    # through the C ABI directly: a null entry for a non-empty variable, a bad dtype, a null list
    import ctypes as C
    from paper_2004_13336_amd._lib import AdamHP, lib
    hp = AdamHP(1e-3, 0.9, 0.999, 1e-8, 0.0)
    P = lambda t: C.c_void_p(t.data_ptr())
    good = (C.c_void_p * 3)(full[0].data_ptr(), full[1].data_ptr(), None)
    bad = (C.c_void_p * 3)(full[0].data_ptr(), None, None)
    call = lib().shard_update_adam_full_grads
    assert call(plan.handle, 0, P(w), good, 0, P(m), P(v), None, C.byref(hp), 1, None) == 0
    assert call(plan.handle, 0, P(w), bad, 0, P(m), P(v), None, C.byref(hp), 1, None) == -1
    assert call(plan.handle, 0, P(w), good, 7, P(m), P(v), None, C.byref(hp), 1, None) == -1
    assert call(plan.handle, 0, P(w), None, 0, P(m), P(v), None, C.byref(hp), 1, None) == -1
    assert call(plan.handle, 0, C.c_void_p(w.data_ptr() + 4), good, 0, P(m), P(v), None, C.byref(hp), 1, None) == -3
    assert call(plan.handle, 0, P(w), good, 0, P(m), P(v), None, C.byref(hp), 0, None) == -1       # step < 1
    torch.cuda.synchronize()
    plan.free()
