"""Pins for oracle/formatting.py."""
import os
import random

import numpy as np
import pytest
import torch

from oracle import make_plan, shard_format, unshard_format, f32_to_bf16_bits, bf16_bits_to_f32
from workloads import random_bits_u32

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "bf16_rounding.txt")


def _bits(seed, numel):
    return [random_bits_u32(seed, i, n).view(np.float32) for i, n in enumerate(numel)]


def _same_bits(a, b):
    return a.dtype == b.dtype and a.shape == b.shape and np.array_equal(a.view(np.uint8), b.view(np.uint8))


@pytest.mark.parametrize("align", [1, 4, 8, 64])
def test_round_trip_random_bit_patterns(align):
    rnd = random.Random(align)
    for N in [1, 2, 3, 4, 7, 8, 16, 31, 32, 33, 64, 100, 128, 129, 130]:
        numel = [rnd.choice([0, 1, 2, N - 1, N, N + 1, 17, 255, 256, 257, 1031, 4096]) for _ in range(6)]
        flats = _bits(100 + N, numel)
        p = make_plan(numel, N, align)
        gathered = np.stack([shard_format(p, r, flats) for r in range(N)])
        back = unshard_format(p, gathered)
        for a, b in zip(flats, back):
            assert _same_bits(a, b)


def test_single_replica_no_align_is_plain_concatenation():
    numel = [5, 0, 12, 1, 33]
    flats = _bits(3, numel)
    p = make_plan(numel, 1, 1)
    assert _same_bits(shard_format(p, 0, flats), np.concatenate(flats))


def test_against_the_layout_equation_element_by_element():
    """shard_r[off_i + k] = flat_i[r L_i + k] if that index exists, else +0.0 (pure-Python loops)."""
    for N, align, numel in [(3, 1, [10, 1, 0, 7]), (4, 4, [17, 64, 5]), (5, 8, [100, 3, 41])]:
        flats = _bits(N, numel)
        p = make_plan(numel, N, align)
        for r in range(N):
            got = shard_format(p, r, flats).view(np.uint32)
            pos = 0
            for i, n in enumerate(numel):
                Li = -(-(-(-n // N)) // align) * align
                for k in range(Li):
                    j = r * Li + k
                    want = int(flats[i].view(np.uint32)[j]) if j < n else 0
                    assert int(got[pos + k]) == want
                pos += Li
            assert pos == got.size


def test_padding_is_positive_zero_bits_and_sits_at_the_tail():
    numel = [10, 3]
    p = make_plan(numel, 4, 4)                 # L = [4, 4]; variable 0 fills replicas 0..2 (4,4,2), variable 1 only replica 0
    flats = [np.full(10, -1.5, np.float32), np.full(3, 2.5, np.float32)]
    s2 = shard_format(p, 2, flats).view(np.uint32)
    assert list(s2) == [0xBFC00000, 0xBFC00000, 0, 0, 0, 0, 0, 0]
    s3 = shard_format(p, 3, flats).view(np.uint32)
    assert not s3.any()


def test_format_reads_only_its_own_piece():
    # Section 4.1: the pad is fused into the slice, nothing outside replica r's piece matters.
    numel = [40, 9]
    p = make_plan(numel, 4, 1)
    flats = _bits(11, numel)
    base = shard_format(p, 1, flats)
    poked = [f.copy() for f in flats]
    poked[0][:10] = 7.0; poked[0][20:] = 7.0       # replica 1 owns [10, 20) of variable 0
    poked[1][:3] = 7.0; poked[1][6:] = 7.0         # and [3, 6) of variable 1
    assert _same_bits(base, shard_format(p, 1, poked))


def test_unshard_ignores_pad_contents():
    numel = [10, 3]
    p = make_plan(numel, 4, 4)
    flats = _bits(5, numel)
    gathered = np.stack([shard_format(p, r, flats) for r in range(4)])
    dirty = gathered.copy()
    for r in range(4):
        for i in range(2):
            real = p.real_count(i, r)
            dirty[r, p.off[i] + real:p.off[i] + p.L[i]] = np.float32(123.0)
    for a, b in zip(flats, unshard_format(p, dirty)):
        assert _same_bits(a, b)


def test_bf16_rounding_hand_worked_cases():
    with open(GOLDEN) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    src = np.array([int(a, 16) for a, _ in rows], dtype=np.uint32).view(np.float32)
    want = np.array([int(b, 16) for _, b in rows], dtype=np.uint16)
    assert np.array_equal(f32_to_bf16_bits(src), want)


def test_bf16_rounding_matches_torch_on_random_patterns():
    x = random_bits_u32(9, 0, 200000).view(np.float32)
    x = np.concatenate([x, np.array([0.0, -0.0, np.inf, -np.inf, 1e-45, -1e-45, 3.3895e38], np.float32)])
    finite_or_inf = ~np.isnan(x)
    got = f32_to_bf16_bits(x)
    ref = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got[finite_or_inf], ref[finite_or_inf])
    back = bf16_bits_to_f32(got)
    assert np.isnan(back[~finite_or_inf]).all()                       # NaN stays NaN
    assert np.array_equal(got[~finite_or_inf] >> 15, x.view(np.uint32)[~finite_or_inf] >> 31)  # with its sign
    # widening is exact
    assert np.array_equal(bf16_bits_to_f32(ref[finite_or_inf]),
                          torch.from_numpy(ref[finite_or_inf].view(np.int16).copy()).view(torch.bfloat16).float().numpy())


def test_bf16_format_variants_round_trip():
    numel = [37, 0, 1000, 5]
    N = 3
    p = make_plan(numel, N, 8)
    flats = [np.random.default_rng(i).standard_normal(n).astype(np.float32) for i, n in enumerate(numel)]
    g16 = np.stack([shard_format(p, r, flats, dst="bf16") for r in range(N)])
    assert g16.dtype == np.uint16
    back16 = unshard_format(p, g16)
    for a, b in zip(flats, back16):
        assert np.array_equal(f32_to_bf16_bits(a), b)
    # converting while unsharding gives the same as converting the full tensor
    g32 = np.stack([shard_format(p, r, flats) for r in range(N)])
    for a, b in zip(flats, unshard_format(p, g32, dst="bf16")):
        assert np.array_equal(f32_to_bf16_bits(a), b)
