"""GPU parity of shard_format / unshard_format against the oracle: bit-exact."""
import random

import numpy as np
import pytest
import torch

import oracle
import paper_2004_13336_amd as su
from helpers import DEV, same_bits, to_dev, to_host
from workloads import CONFIGS, random_bits_u32

pytestmark = pytest.mark.gpu

CANARY = 0x5A


def _bit_tensors(seed, numel, dtype):
    """Host arrays of arbitrary bit patterns: float32 (as float32 arrays) or bf16 (uint16)."""
    out = []
    for i, n in enumerate(numel):
        bits = random_bits_u32(seed, i, n)
        out.append(bits.view(np.float32) if dtype == "f32" else (bits & 0xFFFF).astype(np.uint16))
    return out


def _guarded(nbytes):
    """A device byte buffer with canary bands before and after the payload."""
    band = 256
    buf = torch.full((nbytes + 2 * band,), CANARY, dtype=torch.uint8, device=DEV)
    return buf, buf[band:band + nbytes], band


def _bands_intact(buf, band, nbytes):
    return bool((buf[:band] == CANARY).all()) and bool((buf[band + nbytes:] == CANARY).all())


CASES = [
    # (numel, N, align)
    ([1000, 37, 0, 8, 4099, 1], 3, 8),
    ([5, 6, 7, 64, 1001, 3, 0, 20000], 6, 8),
    ([2, 1024, 30522, 513], 8, 8),
    ([64, 64, 9000], 32, 8),                # replicas whose pieces are all padding
    ([100, 33, 7], 4, 1),                   # element-wise path: pieces not 16-byte aligned
    ([100, 33, 4097], 5, 4),
    ([12345, 8], 1, 8),
    ([70000], 2, 64),
    ([], 4, 8),
    ([0, 0], 4, 8),
    ([1024, 300000, 30522, 2, 70001], 2048, 8),   # thousands of replicas: pieces of 8 to 152 slots, most of them padding
    ([5000, 333, 40000], 1000, 1),                # the same without alignment (5-, 1- and 40-slot pieces)
    ([9000, 16], 257, 16),
    ([3000000, 100, 64, 7, 50000, 1000000], 64, 8),   # variable-by-variable walk with pieces of many chunks among tiny ones
]


@pytest.mark.parametrize("numel,N,align", CASES)
@pytest.mark.parametrize("src,dst", [("f32", "f32"), ("bf16", "bf16"), ("f32", "bf16"), ("bf16", "f32")])
def test_format_and_unshard_match_oracle(numel, N, align, src, dst):
    print("case", numel, N, align, src, dst, flush=True)
    oplan = oracle.make_plan(numel, N, align)
    plan = su.shard_plan_bind(su.shard_plan(numel, N, align))
    flats = _bit_tensors(11, numel, src)
    if src == "f32" and dst == "bf16":
        # NaN payloads are quieted by the conversion on both sides identically; keep them in.
        pass
    dev_full = [to_dev(f) for f in flats]
    tdt = torch.float32 if dst == "f32" else torch.bfloat16
    esz = 4 if dst == "f32" else 2
    gathered_ref = np.stack([oracle.shard_format(oplan, r, flats, dst=dst) for r in range(N)]) if oplan.S else None
    # one guarded, separately allocated (16-byte aligned) output per replica
    rows = []
    for r in range(N):
        buf, payload, band = _guarded(oplan.S * esz)
        out = payload.view(tdt) if oplan.S else torch.empty(0, dtype=tdt, device=DEV)
        su.shard_format(plan, r, dev_full, out)
        torch.cuda.synchronize()
        assert _bands_intact(buf, band, oplan.S * esz)
        if oplan.S:
            assert same_bits(to_host(out), gathered_ref[r]), r
        rows.append(out)
    gathered = torch.stack(rows).contiguous()
    # reverse: restore the full tensors (in dst dtype) and compare with the oracle's unformat
    if oplan.S:
        want_full = oracle.unshard_format(oplan, gathered_ref)
        outs, bufs = [], []
        for n in numel:
            b, p, bd = _guarded(n * esz)
            bufs.append((b, bd, n * esz))
            outs.append(p.view(tdt))
        su.unshard_format(plan, gathered, outs)
        torch.cuda.synchronize()
        for (b, bd, nb), o, w in zip(bufs, outs, want_full):
            assert _bands_intact(b, bd, nb)
            assert same_bits(to_host(o), w)
    plan.free()


@pytest.mark.parametrize("numel,N,align", [([1000, 37, 4099], 3, 8), ([100, 33, 7], 4, 1),
                                          ([1024, 300000, 30522, 2, 70001], 2048, 8),      # variable-by-variable walk
                                          ([5000, 333, 40000], 1000, 1), ([9000, 16], 257, 16)])
@pytest.mark.parametrize("src,dst", [("f32", "bf16"), ("bf16", "f32")])
def test_unshard_converting_between_element_types(numel, N, align, src, dst):
    """float32 shards restored as bfloat16 tensors (rounded to nearest even) and bfloat16 shards as float32
    tensors, on plans of either walk; bit patterns include NaN payloads, infinities and -0.0."""
    oplan = oracle.make_plan(numel, N, align)
    plan = su.shard_plan_bind(su.shard_plan(numel, N, align))
    flats = _bit_tensors(29, numel, src)
    gathered = np.stack([oracle.shard_format(oplan, r, flats) for r in range(N)])
    sdt, ddt = (torch.float32, torch.bfloat16) if src == "f32" else (torch.bfloat16, torch.float32)
    esz = 2 if dst == "bf16" else 4
    outs, bufs = [], []
    for n in numel:
        b, p, bd = _guarded(n * esz)
        bufs.append((b, bd, n * esz))
        outs.append(p.view(ddt))
    rows = torch.empty((N, max(oplan.S, 1)), dtype=sdt, device=DEV)[:, :oplan.S]
    rows.copy_(to_dev(gathered))
    su.unshard_format(plan, rows, outs)
    torch.cuda.synchronize()
    for (b, bd, nb), o, w in zip(bufs, outs, oracle.unshard_format(oplan, gathered, dst=dst)):
        assert _bands_intact(b, bd, nb)
        assert same_bits(to_host(o), w)
    plan.free()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_unshard_reads_strided_rows(dtype):
    """Rows of the gathered buffer may be spaced further apart than S (128-byte aligned rows)."""
    numel, N = [1000, 37, 4099, 20011], 5
    oplan = oracle.make_plan(numel, N, 8)
    plan = su.shard_plan_bind(su.shard_plan(numel, N, 8))
    flats = _bit_tensors(17, numel, dtype)
    ref = np.stack([oracle.shard_format(oplan, r, flats) for r in range(N)])
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    for stride in (oplan.S + 8, oplan.S + 9, None):          # vector path, element-wise path, gathered_empty
        if stride is None:
            gathered = su.gathered_empty(plan, tdt)
            assert gathered.data_ptr() % 128 == 0 and (gathered.stride(0) * gathered.element_size()) % 128 == 0
        else:
            gathered = torch.zeros((N, stride), dtype=tdt, device=DEV)[:, :oplan.S]
        gathered.copy_(to_dev(ref))
        outs = [torch.zeros(n, dtype=tdt, device=DEV) for n in numel]
        su.unshard_format(plan, gathered, outs)
        for o, f in zip(outs, flats):
            assert same_bits(to_host(o), f)
    # rows closer together than S are refused
    import ctypes as C
    arr = (C.c_void_p * len(numel))(*[o.data_ptr() for o in outs])
    assert su.lib().unshard_format(plan.handle, C.c_void_p(gathered.data_ptr()), oplan.S - 8, 0, arr, 0, None) == -1
    plan.free()


def test_misaligned_full_tensors_take_the_elementwise_path():
    numel, N = [1000, 4099, 64], 4
    oplan = oracle.make_plan(numel, N, 8)
    plan = su.shard_plan_bind(su.shard_plan(numel, N, 8))
    flats = _bit_tensors(5, numel, "f32")
    _check_with_shifted_tensors(numel, N, oplan, plan, flats, shifted=(0, 1, 2))     # every tensor misaligned
    _check_with_shifted_tensors(numel, N, oplan, plan, flats, shifted=(1,))          # only the middle one


def _check_with_shifted_tensors(numel, N, oplan, plan, flats, shifted):
    # a shifted tensor starts 4 bytes past a 16-byte boundary
    backing = [torch.empty(n + 4, dtype=torch.float32, device=DEV) for n in numel]
    views = [b[1:1 + n] if i in shifted else b[:n] for i, (b, n) in enumerate(zip(backing, numel))]
    for i, (v, f) in enumerate(zip(views, flats)):
        v.copy_(torch.from_numpy(f))
        assert (v.data_ptr() % 16 != 0) == (i in shifted)
    out = torch.empty(oplan.S, dtype=torch.float32, device=DEV)
    for r in range(N):
        su.shard_format(plan, r, views, out)
        assert same_bits(to_host(out), oracle.shard_format(oplan, r, flats))
    gathered = to_dev(np.stack([oracle.shard_format(oplan, r, flats) for r in range(N)]))
    for v in views:
        v.zero_()
    su.unshard_format(plan, gathered, views)
    for v, f in zip(views, flats):
        assert same_bits(to_host(v), f)


def test_pointer_table_cache_survives_alternating_tensor_sets():
    numel, N = [300, 5000], 2
    oplan = oracle.make_plan(numel, N, 8)
    plan = su.shard_plan_bind(su.shard_plan(numel, N, 8))
    sets = [[to_dev(f) for f in _bit_tensors(s, numel, "f32")] for s in range(6)]   # more sets than cache slots
    host = [_bit_tensors(s, numel, "f32") for s in range(6)]
    out = torch.empty(oplan.S, dtype=torch.float32, device=DEV)
    order = [0, 1, 0, 2, 3, 4, 5, 0, 5, 1, 1, 3]
    for s in order:
        su.shard_format(plan, 1, sets[s], out)
        assert same_bits(to_host(out), oracle.shard_format(oplan, 1, host[s]))


def test_runtime_argument_errors():
    plan = su.shard_plan(([100, 8]), 2)
    t = [torch.zeros(100, device=DEV), torch.zeros(8, device=DEV)]
    out = torch.zeros(plan.S, device=DEV)
    with pytest.raises(su.ShardError) as e:
        su.shard_format(plan, 0, t, out)           # not bound
    assert e.value.status == -5
    su.shard_plan_bind(plan)
    with pytest.raises(su.ShardError) as e:
        su.shard_format(plan, 2, t, out)           # replica id out of range
    assert e.value.status == -1
    with pytest.raises(ValueError):
        su.shard_format(plan, 0, t, out[:-1])      # output too small: refused before any launch
    with pytest.raises(ValueError):
        su.shard_format(plan, 0, [t[0], t[1][:-1]], out)
    with pytest.raises(su.ShardError) as e:
        su.shard_format(plan, 0, t, torch.zeros(plan.S + 1, device=DEV)[1:])   # misaligned shard buffer
    assert e.value.status == -3
    small = torch.empty(16, dtype=torch.uint8, device=DEV)
    with pytest.raises(su.ShardError) as e:
        su.shard_plan_bind(plan, small)
    assert e.value.status == -2


@pytest.mark.parametrize("name,N,replicas", [("bert_large", 8, (0, 7)), ("bert_large", 64, (0, 63, 31)),
                                             ("resnet50", 32, (0, 31)), ("resnet50", 1, (0,))])
def test_full_size_format_round_trip(name, N, replicas):
    """At the benchmark's sizes: sampled replicas bit-exact against the oracle, then the whole
    gathered buffer unsharded and compared with the inputs."""
    cfg = [c for c in CONFIGS if c.name == name][0]
    print("full-size format", name, N, flush=True)
    numel = cfg.numel
    oplan = oracle.make_plan(numel, N, 8)
    plan = su.shard_plan_bind(su.shard_plan(numel, N, 8))
    flats = _bit_tensors(cfg.seed, numel, "f32")
    dev_full = [to_dev(f) for f in flats]
    gathered = torch.empty((N, oplan.S), dtype=torch.float32, device=DEV)
    for r in range(N):
        su.shard_format(plan, r, dev_full, gathered[r])
    for r in replicas:
        assert same_bits(to_host(gathered[r]), oracle.shard_format(oplan, r, flats)), r
    # all replicas in one pass (at 64 replicas of the 340 M model: large pieces replica by replica, small ones
    # variable by variable): the same bits as replica after replica, in rows 128 bytes apart too
    # ... and in either order of the work items, whichever the plan or its measurement would pick
    both = su.gathered_empty(plan)
    outs = [torch.empty(n, dtype=torch.float32, device=DEV) for n in numel]
    for walk in ("auto", "by_replica", "by_variable"):
        su.shard_plan_set_copy_walk(plan, walk)
        both.fill_(7.0)
        su.shard_format_all(plan, dev_full, both)
        assert torch.equal(both.view(torch.int32), gathered.view(torch.int32)), walk
        for o in outs:
            o.fill_(7.0)
        su.unshard_format(plan, gathered, outs)
        for i, (o, f) in enumerate(zip(outs, flats)):
            assert same_bits(to_host(o), f), (walk, i)
    del both
    plan.free()


def test_full_size_converting_copies_bert_large_8_replicas():
    """The converting copies at the benchmark's size (340 M parameters, 8 replicas: the stages
    unshard_format_f32_to_bf16 and shard_format_bf16_to_f32 time exactly these launches): float32 shards restored
    as bfloat16 tensors, bfloat16 tensors formatted into float32 shards, float32 tensors into a bfloat16
    gathered buffer; every element against the oracle's conversion of the same bits."""
    cfg = [c for c in CONFIGS if c.name == "bert_large"][0]
    N, numel = 8, cfg.numel
    print("full-size converting copies", cfg.name, N, flush=True)
    oplan = oracle.make_plan(numel, N, 8)
    plan = su.shard_plan_bind(su.shard_plan(numel, N, 8))
    flats = _bit_tensors(cfg.seed + 1, numel, "f32")              # NaN payloads, infinities, denormals included
    dev_full = [to_dev(f) for f in flats]
    gathered = su.gathered_empty(plan)
    su.shard_format_all(plan, dev_full, gathered)
    # float32 gathered buffer -> bfloat16 full tensors, in both orders of the work items
    want16 = [oracle.f32_to_bf16_bits(f) for f in flats]
    outs16 = [torch.empty(n, dtype=torch.bfloat16, device=DEV) for n in numel]
    for walk in ("by_replica", "by_variable"):
        su.shard_plan_set_copy_walk(plan, walk)
        for o in outs16:
            o.view(torch.int16).fill_(0x5A5A)
        su.unshard_format(plan, gathered, outs16)
        for i, (o, w) in enumerate(zip(outs16, want16)):
            assert same_bits(to_host(o), w), (walk, i)
    # float32 full tensors -> bfloat16 gathered buffer: row r is the oracle's shard r, converted
    rows16 = torch.empty((N, oplan.S), dtype=torch.bfloat16, device=DEV)
    for walk in ("by_replica", "by_variable"):
        su.shard_plan_set_copy_walk(plan, walk)
        rows16.view(torch.int16).fill_(0x5A5A)
        su.shard_format_all(plan, dev_full, rows16)
        for r in (0, 3, 7):
            assert same_bits(to_host(rows16[r]), oracle.shard_format(oplan, r, flats, dst="bf16")), (walk, r)
    # one replica at a time gives the same rows
    one = torch.empty(oplan.S, dtype=torch.bfloat16, device=DEV)
    for r in (0, 7):
        su.shard_format(plan, r, dev_full, one)
        assert torch.equal(one.view(torch.int16), rows16[r].view(torch.int16)), r
    # bfloat16 full tensors -> float32 shard
    su.shard_plan_set_copy_walk(plan, "auto")
    out32 = torch.empty(oplan.S, dtype=torch.float32, device=DEV)
    for r in (0, 7):
        su.shard_format(plan, r, outs16, out32)
        assert same_bits(to_host(out32), oracle.shard_format(oplan, r, want16, dst="f32")), r
    plan.free()


def test_formatting_stress_1p5b_128_replicas_bf16():
    """771 variables, 128 replicas: [1600]-element variables leave 13 real + 3 padded slots per
    replica and hundreds of all-padding pieces on the last replicas."""
    cfg = [c for c in CONFIGS if c.name == "lm_1p5b"][0]
    N = 128
    numel = cfg.numel
    oplan = oracle.make_plan(numel, N, 8)
    plan = su.shard_plan_bind(su.shard_plan(numel, N, 8))
    gen = torch.Generator(device=DEV)
    gen.manual_seed(cfg.seed)
    flat_all = torch.randint(-32768, 32767, (cfg.total,), dtype=torch.int16, device=DEV, generator=gen)
    pos, dev_full = 0, []
    for n in numel:
        dev_full.append(flat_all[pos:pos + n].view(torch.bfloat16))    # offsets are multiples of 8 elements
        pos += n
    host_all = flat_all.cpu().numpy().view(np.uint16)
    pos, flats = 0, []
    for n in numel:
        flats.append(host_all[pos:pos + n])
        pos += n
    out = torch.empty(oplan.S, dtype=torch.bfloat16, device=DEV)
    for r in (0, 1, 77, 126, 127):
        su.shard_format(plan, r, dev_full, out)
        assert same_bits(to_host(out), oracle.shard_format(oplan, r, flats)), r
    # whole round trip on the device, checked against the inputs
    gathered = torch.empty((N, oplan.S), dtype=torch.bfloat16, device=DEV)
    for r in range(N):
        su.shard_format(plan, r, dev_full, gathered[r])
    back = torch.zeros(cfg.total, dtype=torch.int16, device=DEV)
    pos, outs = 0, []
    for n in numel:
        outs.append(back[pos:pos + n].view(torch.bfloat16))
        pos += n
    su.unshard_format(plan, gathered, outs)
    assert torch.equal(back, flat_all)
    plan.free()


@pytest.mark.parametrize("numel,N,align", [([1000, 37, 0, 8, 4099, 1], 3, 8), ([64, 64, 9000], 32, 8), ([100, 33, 7], 4, 1),
                                          ([2, 1024, 30522, 513], 8, 8), ([1024, 300000, 30522, 2, 70001], 2048, 8),
                                          ([5000, 333, 40000], 1000, 1),
                                          ([3000000, 100, 64, 7, 50000, 1000000], 64, 8),
                                          ([5000, 2000001, 3, 700000], 100, 4)])
@pytest.mark.parametrize("src,dst", [("f32", "f32"), ("f32", "bf16"), ("bf16", "bf16"), ("bf16", "f32")])
def test_format_all_replicas_in_one_pass(numel, N, align, src, dst):
    """Row r of the output is shard_r, for all r at once (the reduce-scatter input layout)."""
    oplan = oracle.make_plan(numel, N, align)
    plan = su.shard_plan_bind(su.shard_plan(numel, N, align))
    flats = _bit_tensors(23, numel, src)
    dev_full = [to_dev(f) for f in flats]
    tdt = torch.float32 if dst == "f32" else torch.bfloat16
    esz = 4 if dst == "f32" else 2
    ref = np.stack([oracle.shard_format(oplan, r, flats, dst=dst) for r in range(N)])
    # back-to-back rows, with canaries around the whole buffer
    buf, payload, band = _guarded(N * oplan.S * esz)
    out = payload.view(tdt).view(N, oplan.S)
    su.shard_format_all(plan, dev_full, out)
    torch.cuda.synchronize()
    assert _bands_intact(buf, band, N * oplan.S * esz)
    assert same_bits(to_host(out), ref)
    # strided rows: the slots between S and the stride keep their contents
    stride = oplan.S + 24
    wide = torch.full((N, stride), 3.0, dtype=tdt, device=DEV)
    su.shard_format_all(plan, dev_full, wide[:, :oplan.S])
    assert same_bits(to_host(wide[:, :oplan.S].contiguous()), ref)
    assert bool((wide[:, oplan.S:] == 3.0).all())
    plan.free()


@pytest.mark.parametrize("align,src,dst", [(8, "f32", "bf16"), (4, "bf16", "f32")])
def test_format_all_split_walk_with_conversion(align, src, dst):
    """Large enough (2^26 elements) for the plan to split the all-replica formatting: the two big variables
    replica by replica, the small ones variable by variable; with a conversion, and once on the element-wise path."""
    numel, N = [67000000] + [100, 64, 7, 1000] * 50 + [50000, 1200003], 64     # the small ones make the plan leave the replica walk
    oplan = oracle.make_plan(numel, N, align)
    plan = su.shard_plan_bind(su.shard_plan(numel, N, align))
    flats = _bit_tensors(41, numel, src)
    dev_full = [to_dev(f) for f in flats]
    tdt = torch.float32 if dst == "f32" else torch.bfloat16
    rows = torch.full((N, oplan.S + 8), 3.0, dtype=tdt, device=DEV)
    su.shard_format_all(plan, dev_full, rows[:, :oplan.S])
    assert bool((rows[:, oplan.S:] == 3.0).all())
    for r in (0, 1, 31, 62, 63):
        assert same_bits(to_host(rows[r, :oplan.S].contiguous()), oracle.shard_format(oplan, r, flats, dst=dst)), r
    # and back, through the variable-by-variable unshard, into the source type
    back = [torch.empty(n, dtype=torch.float32 if src == "f32" else torch.bfloat16, device=DEV) for n in numel]
    su.unshard_format(plan, rows[:, :oplan.S], back)
    if src == "bf16":                                   # bf16 -> f32 -> bf16 is the identity on every bit pattern but NaN payloads
        for o, f in zip(back, flats):
            a, b = to_host(o), f
            nan = (b & 0x7F80 == 0x7F80) & (b & 0x007F != 0)
            assert np.array_equal(a[~nan], b[~nan])
    plan.free()


def test_format_all_full_size_transformer():
    cfg = [c for c in CONFIGS if c.name == "transformer_big"][0]
    N = 16
    oplan = oracle.make_plan(cfg.numel, N, 8)
    plan = su.shard_plan_bind(su.shard_plan(cfg.numel, N, 8))
    flats = _bit_tensors(cfg.seed, cfg.numel, "f32")
    dev_full = su.FullTensors(plan, [to_dev(f) for f in flats])
    out = su.gathered_empty(plan)
    su.shard_format_all(plan, dev_full, out)
    for r in (0, 7, 15):
        assert same_bits(to_host(out[r]), oracle.shard_format(oplan, r, flats)), r
    back = [torch.empty(n, dtype=torch.float32, device=DEV) for n in cfg.numel]
    su.unshard_format(plan, out, back)
    for o, f in zip(back, flats):
        assert same_bits(to_host(o), f)
    plan.free()


def test_random_plans_whole_model_copies():
    """Seeded random variable lists and replica counts, small pieces and large: shard_format_all against the
    oracle's shards (every row, or a sample of rows where there are thousands) and unshard_format back."""
    rnd = random.Random(2024)
    sizes = [0, 1, 2, 7, 8, 9, 63, 64, 65, 500, 1023, 1024, 1025, 4096, 4100, 30000, 65536, 100003]
    for case in range(24):
        N = rnd.choice([1, 2, 3, 5, 8, 31, 64, 100, 257, 1000, 3001])
        align = rnd.choice([8, 8, 8, 16, 64, 1, 4])
        numel = [rnd.choice(sizes) for _ in range(rnd.randint(1, 7))]
        dtype = rnd.choice(["f32", "bf16"])
        print("random plan", case, N, align, numel, dtype, flush=True)
        oplan = oracle.make_plan(numel, N, align)
        plan = su.shard_plan_bind(su.shard_plan(numel, N, align))
        flats = _bit_tensors(300 + case, numel, dtype)
        dev_full = [to_dev(f) for f in flats]
        tdt = torch.float32 if dtype == "f32" else torch.bfloat16
        if align % 8 == 0:
            rows = su.gathered_empty(plan, tdt)
        else:
            rows = torch.empty((N, max(oplan.S, 1)), dtype=tdt, device=DEV)[:, :oplan.S]
        check = range(N) if N <= 100 else sorted({0, 1, N // 3, N // 2, N - 2, N - 1} | {rnd.randrange(N) for _ in range(10)})
        want = {r: oracle.shard_format(oplan, r, flats) for r in check}
        for walk in ("auto", "by_replica", "by_variable"):           # the plan's own choice, then each order forced
            su.shard_plan_set_copy_walk(plan, walk)
            rows.fill_(3.0)
            su.shard_format_all(plan, dev_full, rows)
            got = to_host(rows.contiguous())
            for r in check:
                assert same_bits(got[r], want[r]), (case, walk, r)
            back = [torch.full((n,), 5.0, dtype=tdt, device=DEV) for n in numel]
            su.unshard_format(plan, rows, back)
            for i, (o, f) in enumerate(zip(back, flats)):
                assert same_bits(to_host(o), f), (case, walk, i)
        plan.free()


def test_plain_copy_measurement_aid():
    plan = su.shard_plan([64], 2)                                   # any plan: it only carries the event records
    src = torch.arange(0, 1 << 20, dtype=torch.int32, device=DEV)
    buf, payload, band = _guarded(src.numel() * 4)
    dst = payload.view(torch.int32)
    su.shard_profile_reset(plan); su.shard_profile_enable(plan, True)
    su.shard_profile_plain_copy(plan, dst, src)
    su.shard_profile_plain_copy(plan, dst[:1000], src[4:1004])     # 4000 bytes, 16-byte aligned ends
    torch.cuda.synchronize()
    assert torch.equal(dst[1000:], src[1000:]) and torch.equal(dst[:1000], src[4:1004]) and _bands_intact(buf, band, src.numel() * 4)
    n, ms = su.shard_profile_read(plan, "plain_copy")
    assert n == 2 and ms > 0.0
    with pytest.raises(su.ShardError) as e:
        su.shard_profile_plain_copy(plan, dst[:1001], src[:1001])   # 4004 bytes
    assert e.value.status == -1
    with pytest.raises(su.ShardError) as e:
        su.shard_profile_plain_copy(plan, dst[:1000], src[1:1001])  # source 4 bytes off a 16-byte boundary
    assert e.value.status == -3
    plan.free()


WALK_CASES = [([30000, 37, 0, 8, 4099, 1, 65536], 3, 8), ([9000, 64, 64], 32, 8), ([100, 33, 7], 4, 1),
              ([20011, 4096, 5], 1, 8)]


@pytest.mark.gpu
@pytest.mark.parametrize("numel,N,align", WALK_CASES)
@pytest.mark.parametrize("src,dst", [("f32", "f32"), ("f32", "bf16"), ("bf16", "f32")])
def test_both_orders_of_the_whole_model_copies_write_the_same_bytes(numel, N, align, src, dst):
    """shard_format_all and unshard_format with the order forced either way against the oracle, on plans
    whose default would be the one and the other."""
    oplan = oracle.make_plan(numel, N, align)
    flats = _bit_tensors(41, numel, src)
    sdt = torch.float32 if src == "f32" else torch.bfloat16
    ddt = torch.float32 if dst == "f32" else torch.bfloat16
    want_rows = np.stack([oracle.shard_format(oplan, r, flats, dst=dst) for r in range(N)])
    src_ref = np.stack([oracle.shard_format(oplan, r, flats) for r in range(N)])
    want_full = oracle.unshard_format(oplan, src_ref, dst=dst)
    for walk in ("by_replica", "by_variable"):
        plan = su.shard_plan_bind(su.shard_plan(numel, N, align))
        su.shard_plan_set_copy_walk(plan, walk)
        full = [to_dev(f) for f in flats]
        expect = walk if (N > 1) else "by_replica"
        assert su.shard_plan_copy_walk(plan, "shard_format_all", full) == expect
        rows = torch.full((N, max(oplan.S, 1)), 7.0, dtype=ddt, device=DEV)[:, :oplan.S]
        su.shard_format_all(plan, full, rows)
        assert same_bits(to_host(rows), want_rows), walk
        src_rows = torch.empty((N, max(oplan.S, 1)), dtype=sdt, device=DEV)[:, :oplan.S]
        src_rows.copy_(to_dev(src_ref))
        outs = [torch.full((n,), 7.0, dtype=ddt, device=DEV) for n in numel]
        su.unshard_format(plan, src_rows, outs)
        for o, w in zip(outs, want_full):
            assert same_bits(to_host(o), w), walk
        plan.free()


@pytest.mark.gpu
def test_tuned_order_is_explicit_deterministic_and_every_copy_is_right():
    """With large pieces the copies go by replica until the caller has the two orders measured for a list of
    tensors: plain calls never time anything and never change order by themselves; the tuning call runs the copy
    for real in both orders, reports what it chose with both times, and later calls with that list keep the choice
    whatever else runs on the stream in between; another list, element type or row stride is untuned again."""
    numel, N = [262144, 100, 131072, 70000, 262144], 4
    oplan = oracle.make_plan(numel, N, 8)
    plan = su.shard_plan_bind(su.shard_plan(numel, N, 8))
    flats = _bit_tensors(43, numel, "f32")
    ref = np.stack([oracle.shard_format(oplan, r, flats) for r in range(N)])
    gathered = su.gathered_empty(plan)
    gathered.copy_(to_dev(ref))
    outs = [torch.zeros(n, device=DEV) for n in numel]
    noise = torch.zeros(1 << 24, device=DEV)
    for k in range(8):                       # untuned calls under a varying load: the order never moves
        for o in outs:
            o.fill_(3.0)
        if k & 1:
            noise.add_(1.0)                  # other work on the stream
        su.unshard_format(plan, gathered, outs)
        torch.cuda.synchronize()
        for o, f in zip(outs, flats):
            assert same_bits(to_host(o), f)
        assert su.shard_plan_copy_walk(plan, "unshard_format", outs, with_times=True) == ("by_replica", (0.0, 0.0))
    for o in outs:
        o.fill_(3.0)
    walk, (ms_rep, ms_var) = su.shard_plan_tune_copy_walk(plan, "unshard_format", gathered, outs)
    torch.cuda.synchronize()
    assert walk in ("by_replica", "by_variable") and ms_rep > 0.0 and ms_var > 0.0
    assert walk == ("by_variable" if ms_var < 0.95 * ms_rep else "by_replica")
    for o, f in zip(outs, flats):            # the tuning call ran the copy for real
        assert same_bits(to_host(o), f)
    assert su.shard_plan_copy_walk(plan, "unshard_format", outs, with_times=True) == (walk, (ms_rep, ms_var))
    for k in range(6):                       # the choice stays, under load or not
        if k & 1:
            noise.add_(1.0)
        su.unshard_format(plan, gathered, outs)
        assert su.shard_plan_copy_walk(plan, "unshard_format", outs) == walk
    torch.cuda.synchronize()
    for o, f in zip(outs, flats):
        assert same_bits(to_host(o), f)
    # the other copy and another list of tensors have not been measured
    assert su.shard_plan_copy_walk(plan, "shard_format_all", outs, with_times=True) == ("by_replica", (0.0, 0.0))
    others = [torch.zeros(n, device=DEV) for n in numel]
    assert su.shard_plan_copy_walk(plan, "unshard_format", others, with_times=True) == ("by_replica", (0.0, 0.0))
    rows = torch.zeros_like(gathered)
    rows.fill_(5.0)
    walk2, times2 = su.shard_plan_tune_copy_walk(plan, "shard_format_all", rows, outs)
    torch.cuda.synchronize()
    assert same_bits(to_host(rows), ref)
    assert su.shard_plan_copy_walk(plan, "shard_format_all", outs, with_times=True) == (walk2, times2)
    # a forced order wins over a tuned one, and tuning then launches nothing
    su.shard_plan_set_copy_walk(plan, "by_variable")
    assert su.shard_plan_tune_copy_walk(plan, "unshard_format", gathered, outs) == ("by_variable", (0.0, 0.0))
    su.shard_plan_set_copy_walk(plan, "auto")
    assert su.shard_plan_copy_walk(plan, "unshard_format", outs) == walk
    # refused while the stream is being captured (it waits for its launches)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        with pytest.raises(su.ShardError) as err:
            su.shard_plan_tune_copy_walk(plan, "unshard_format", gathered, outs)
        su.unshard_format(plan, gathered, outs)
    assert err.value.status == -5
    torch.cuda.synchronize()
    plan.free()
