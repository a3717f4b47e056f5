"""The whole step (format, LAMB, unshard) recorded in a HIP graph: every replay must equal the eager
step bit for bit, with eager work and synchronisations between the replays.  The library's step path
allocates nothing, synchronises nothing and records no memset, so it can be captured as it is."""
import numpy as np
import pytest
import torch

import oracle
import paper_2004_13336_amd as su
from helpers import DEV, f32_hp, same_bits, to_dev, to_host
from workloads import CONFIGS, normal_f32

pytestmark = pytest.mark.gpu

LAMB = f32_hp({"lr": 1e-3, "beta1": 0.9, "beta2": 0.999, "eps": 1e-6, "weight_decay": 0.01})


class State:
    def __init__(self, plan, cfg, r, seed):
        S, N = plan.S, plan.N
        self.full_g = [to_dev(normal_f32(seed, i, "g", n, 1e-2, 1)) for i, n in enumerate(cfg.numel)]
        self.full_w = [torch.zeros(n, dtype=torch.float32, device=DEV) for n in cfg.numel]
        ws = [normal_f32(seed, i, "w", n, 0.02) for i, n in enumerate(cfg.numel)]
        oplan = oracle.make_plan(cfg.numel, N, 8)
        self.gathered = to_dev(np.stack([oracle.shard_format(oplan, q, ws) for q in range(N)]))
        self.g = torch.zeros(S, dtype=torch.float32, device=DEV)
        self.m = torch.zeros(S, dtype=torch.float32, device=DEV)
        self.v = torch.zeros(S, dtype=torch.float32, device=DEV)
        self.w16 = torch.zeros(S, dtype=torch.bfloat16, device=DEV)
        self.other = torch.full((plan.V, 2), 0.25, dtype=torch.float32, device=DEV)
        self.r = r
        self.fused = False

    def step(self, plan):
        r = self.r
        if self.fused:                          # the gradient read in place from the full tensors
            su.shard_update_lamb_full_grads(plan, r, self.gathered[r], self.full_g, self.m, self.v, LAMB, 5,
                                            other_replicas_sumsq=self.other, w_bf16_out=self.w16)
        else:
            su.shard_format(plan, r, self.full_g, self.g)
            su.shard_update_lamb(plan, r, self.gathered[r], self.g, self.m, self.v, LAMB, 5,
                                 other_replicas_sumsq=self.other, w_bf16_out=self.w16)
        su.unshard_format(plan, self.gathered, self.full_w)

    def snapshot(self):
        return [to_host(t) for t in (self.gathered, self.m, self.v, self.w16, torch.cat(self.full_w))]


@pytest.mark.parametrize("fused", [False, True])
def test_step_captured_in_a_graph_replays_like_eager(fused):
    """fused: the captured step reads the gradient from the full tensors; the eager one it is compared with
    formats it first (the two routes give the same bits)."""
    cfg = [c for c in CONFIGS if c.name == "tiny"][0]
    N, r = 4, 1
    plan = su.shard_plan_bind(su.shard_plan(cfg.numel, N, 8))
    eager, graphed = State(plan, cfg, r, 91), State(plan, cfg, r, 91)
    graphed.fused = fused
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        graphed.step(plan)                      # warm-up on the capture stream: pointer tables become resident
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        graphed.step(plan)
    torch.cuda.synchronize()
    # both states restart from the same point: the warm-up and the capture pass moved `graphed`
    fresh = State(plan, cfg, r, 91)
    for dst, src in ((graphed, fresh), (eager, fresh)):
        dst.gathered.copy_(src.gathered); dst.m.zero_(); dst.v.zero_(); dst.w16.zero_(); dst.g.zero_()
        for a in dst.full_w:
            a.zero_()
    torch.cuda.synchronize()
    previous = None
    for k in range(4):
        graph.replay()
        torch.cuda.synchronize()
        eager.step(plan)                        # eager work of the same library between the replays
        torch.cuda.synchronize()
        a, b = graphed.snapshot(), eager.snapshot()
        assert all(same_bits(x, y) for x, y in zip(a, b)), "replay %d differs from the eager step" % k
        if previous is not None:
            assert not same_bits(a[0], previous[0])          # the state does move from replay to replay
        previous = a
    plan.free()


def test_two_plans_on_two_streams_do_not_disturb_each_other():
    # the library keeps no state outside a plan: two plans driven from two streams, launches interleaved
    # without synchronisation in between, give what each gives alone
    cfg = [c for c in CONFIGS if c.name == "tiny"][0]
    plans = [su.shard_plan_bind(su.shard_plan(cfg.numel, 4, 8)), su.shard_plan_bind(su.shard_plan(cfg.numel[::-1], 3, 8))]

    class Cfg:                                   # the second plan sees the variables in reverse order
        def __init__(self, numel):
            self.numel = numel
    cfgs = [Cfg(list(cfg.numel)), Cfg(list(cfg.numel[::-1]))]
    alone = []
    for plan, c, r in zip(plans, cfgs, (1, 2)):
        st = State(plan, c, r, 93)
        for _ in range(3):
            st.step(plan)
        torch.cuda.synchronize()
        alone.append(st.snapshot())
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    states = [State(plan, c, r, 93) for plan, c, r in zip(plans, cfgs, (1, 2))]
    torch.cuda.synchronize()
    for _ in range(3):
        for st, plan, s in zip(states, plans, streams):
            with torch.cuda.stream(s):
                st.step(plan)
    torch.cuda.synchronize()
    for st, want in zip(states, alone):
        assert all(same_bits(a, b) for a, b in zip(st.snapshot(), want))
    for plan in plans:
        plan.free()


AF = f32_hp({"eps1": 1e-30, "eps2": 1e-3, "clip_threshold": 1.0, "decay_exponent": 0.8, "max_rho": 1e-2})
LARS = f32_hp({"lr": 0.1, "mu": 0.9, "weight_decay": 5e-5, "trust_coeff": 1e-3, "eps": 1e-9})


@pytest.mark.parametrize("optimizer", ["adafactor", "lars", "adam_full_grads"])
def test_other_optimizers_captured_in_a_graph_replay_like_eager(optimizer):
    """The same check for the steps the first test does not cover: Adafactor on a row plan (six kernels, tables kept
    in the workspace between them), LARS, and Adam reading the full gradients; format and unshard around each."""
    rows, cols, N, r = [96, 1, 40, 7], [128, 200, 64, 33], 4, 2
    numel = [a * b for a, b in zip(rows, cols)]

    def make_plan():
        return su.shard_plan_bind(su.shard_plan_rows(rows, cols, N, 8) if optimizer == "adafactor"
                                  else su.shard_plan(numel, N, 8))
    # a plan of its own for each of the two: a recorded graph reads the pointer tables that were resident at
    # capture time, and the two states together pass more than four lists of tensors
    plans = [make_plan(), make_plan()]
    S = plans[0].S
    _, _, total_rows, total_cols = su.shard_plan_rowcol_layout(plans[0]) if optimizer == "adafactor" else (0, 0, 1, 1)

    class St:
        def __init__(self, plan):
            self.plan = plan
            self.full_g = [to_dev(normal_f32(95, i, "g", n, 1e-2, 1)) for i, n in enumerate(numel)]
            self.full_w0 = [to_dev(normal_f32(95, i, "w", n, 0.02)) for i, n in enumerate(numel)]
            self.full_w = [torch.zeros(n, device=DEV) for n in numel]
            self.gathered = su.gathered_empty(plan).zero_()
            self.g = torch.zeros(S, device=DEV)
            self.m = torch.zeros(S, device=DEV)
            self.v = torch.zeros(S, device=DEV)
            self.R = torch.zeros(total_rows, device=DEV)
            self.C = torch.zeros(total_cols, device=DEV)
            self.reset()

        def reset(self):
            plan = self.plan
            su.shard_format_all(plan, self.full_w0, self.gathered)
            for t in (self.g, self.m, self.v, self.R, self.C, *self.full_w):
                t.zero_()

        def step(self):
            plan, w = self.plan, self.gathered[r]
            if optimizer == "adam_full_grads":
                su.shard_update_adam_full_grads(plan, r, w, self.full_g, self.m, self.v, LAMB, 3)
            else:
                su.shard_format(plan, r, self.full_g, self.g)
                if optimizer == "adafactor":
                    su.shard_update_adafactor(plan, r, w, self.g, self.R, self.C, AF, 3)
                else:
                    su.shard_update_lars(plan, r, w, self.g, self.m, LARS)
            su.unshard_format(plan, self.gathered, self.full_w)

        def snapshot(self):
            return [to_host(t) for t in (self.gathered, self.m, self.v, self.R, self.C, torch.cat(self.full_w))]

    eager, graphed = St(plans[0]), St(plans[1])
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        graphed.step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        graphed.step()
    torch.cuda.synchronize()
    graphed.reset()
    torch.cuda.synchronize()
    previous = None
    for k in range(4):
        graph.replay()
        torch.cuda.synchronize()
        eager.step()
        torch.cuda.synchronize()
        a, b = graphed.snapshot(), eager.snapshot()
        assert all(same_bits(x, y) for x, y in zip(a, b)), "%s: replay %d differs from the eager step" % (optimizer, k)
        if previous is not None:
            assert not same_bits(a[0], previous[0])
        previous = a
    for plan in plans:
        plan.free()


def test_tables_a_recorded_graph_reads_are_never_overwritten():
    """A graph reads the pointer tables its calls used at capture time.  Other lists of tensors passed to the same
    plan afterwards share the remaining slots; once every slot belongs to a graph a new list is refused, until the
    caller releases them."""
    cfg = [c for c in CONFIGS if c.name == "tiny"][0]
    N, r = 4, 1
    plan, ref_plan = su.shard_plan_bind(su.shard_plan(cfg.numel, N, 8)), su.shard_plan_bind(su.shard_plan(cfg.numel, N, 8))
    graphed, eager = State(plan, cfg, r, 97), State(ref_plan, cfg, r, 97)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        graphed.step(plan)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        graphed.step(plan)                      # reserves the tables of its gradient and weight tensors
    torch.cuda.synchronize()
    fresh = State(ref_plan, cfg, r, 97)
    for dst in (graphed, eager):
        dst.gathered.copy_(fresh.gathered); dst.m.zero_(); dst.v.zero_(); dst.w16.zero_(); dst.g.zero_()
        for a in dst.full_w:
            a.zero_()
    others = [[torch.ones(n, device=DEV) * k for n in cfg.numel] for k in range(5)]
    scratch = torch.zeros(plan.S, device=DEV)
    for k in range(3):
        for lst in others:                      # five more lists through the two slots that are left
            su.shard_format(plan, r, lst, scratch)
        graph.replay()
        eager.step(ref_plan)
        torch.cuda.synchronize()
        assert all(same_bits(x, y) for x, y in zip(graphed.snapshot(), eager.snapshot())), k
    # a second graph takes the other two slots
    second = State(plan, cfg, r, 98)
    with torch.cuda.stream(side):
        second.step(plan)
    torch.cuda.synchronize()
    graph2 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph2, stream=side):
        second.step(plan)
    torch.cuda.synchronize()
    with pytest.raises(su.ShardError) as err:
        su.shard_format(plan, r, others[0], scratch)
    assert err.value.status == -5
    su.shard_format(plan, r, graphed.full_g, scratch)        # lists that are resident still work
    graph.replay(); graph2.replay()
    torch.cuda.synchronize()
    del graph, graph2
    su.shard_plan_release_captured_tables(plan)
    su.shard_format(plan, r, others[0], scratch)
    torch.cuda.synchronize()
    assert bool((scratch[: 8] == 0.0).all())                 # others[0] is all zeros
    plan.free(); ref_plan.free()


def test_a_list_first_seen_during_capture_is_safe_for_eager_calls_and_replays():
    """No eager warm-up: the plan sees the lists of full tensors for the first time while the stream is being
    captured, so their pointer tables are uploaded by kernels that were only recorded.  Eager calls with the
    same lists before the first replay must not trust those tables (they upload their own), and the graph must
    carry its uploads: every replay equals the eager step."""
    cfg = [c for c in CONFIGS if c.name == "tiny"][0]
    N, r = 4, 1
    plan, ref_plan = su.shard_plan_bind(su.shard_plan(cfg.numel, N, 8)), su.shard_plan_bind(su.shard_plan(cfg.numel, N, 8))
    # poison the plan's pointer-table slots with other tensors, so that a stale table would not go unnoticed
    decoys = [[torch.full((n,), 9.0, device=DEV) for n in cfg.numel] for _ in range(4)]
    tmp = torch.zeros(plan.S, device=DEV)
    for lst in decoys:
        su.shard_format(plan, r, lst, tmp)
    graphed, eager = State(plan, cfg, r, 99), State(ref_plan, cfg, r, 99)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        graphed.step(plan)                      # first sight of graphed.full_g and graphed.full_w
    torch.cuda.synchronize()
    # eager calls with the same two lists, before any replay
    want = torch.zeros(plan.S, device=DEV)
    su.shard_format(ref_plan, r, graphed.full_g, want)
    su.shard_format(plan, r, graphed.full_g, tmp)
    torch.cuda.synchronize()
    assert torch.equal(tmp, want)
    su.unshard_format(plan, graphed.gathered, graphed.full_w)
    su.unshard_format(ref_plan, eager.gathered, eager.full_w)
    torch.cuda.synchronize()
    assert same_bits(to_host(torch.cat(graphed.full_w)), to_host(torch.cat(eager.full_w)))
    for a in graphed.full_w + eager.full_w:
        a.zero_()
    torch.cuda.synchronize()
    for k in range(3):
        graph.replay()
        torch.cuda.synchronize()
        eager.step(ref_plan)
        torch.cuda.synchronize()
        assert all(same_bits(x, y) for x, y in zip(graphed.snapshot(), eager.snapshot())), "replay %d" % k
    # every slot is now taken (two reserved by the graph, two by the eager uploads of the same lists): once the
    # graph is gone and its tables are released, other lists fit again
    del graph
    su.shard_plan_release_captured_tables(plan)
    for lst in decoys:
        su.shard_format(plan, r, lst, tmp)
    torch.cuda.synchronize()
    assert bool((tmp[:8] == 9.0).all())
    plan.free(); ref_plan.free()
