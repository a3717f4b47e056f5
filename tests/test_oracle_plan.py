"""Pins for oracle/plan.py: the paper's worked shape examples, invariants, brute force."""
import os
import random

import pytest

from oracle import make_plan

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "plan_examples.txt")


def _golden_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(tuple(int(x) for x in line.split()))
    return rows


@pytest.mark.parametrize("numel,N,align,piece,pad", _golden_rows())
def test_paper_shape_examples(numel, N, align, piece, pad):
    p = make_plan([numel], N, align)
    assert p.L[0] == piece
    assert p.N * p.S - numel == pad


def test_flat_format_pads_no_more_than_the_papers_row_format():
    # Section 4.1: [9,256,256] -> [10,256,256] pads one 256x256 row; combining every dim pads less.
    p = make_plan([3 * 3 * 256 * 256], 10, 1)
    assert 0 <= p.N * p.L[0] - p.numel[0] <= 256 * 256


SIZES = [0, 1, 2, 3, 7, 8, 9, 63, 64, 65, 127, 128, 129, 1000, 1023, 1024, 1025, 4099, 65537]


@pytest.mark.parametrize("align", [1, 4, 8, 64])
def test_invariants_random_lists(align):
    rnd = random.Random(7 + align)
    for _ in range(60):
        N = rnd.randint(1, 130)
        numel = [rnd.choice(SIZES + [N - 1, N, N + 1, 2 * N + 1]) for _ in range(rnd.randint(1, 12))]
        p = make_plan(numel, N, align)
        assert p.S == sum(p.L)
        pos = 0
        for i, n in enumerate(numel):
            assert p.off[i] == pos                      # pieces are packed back to back, caller's order
            pos += p.L[i]
            assert p.L[i] % align == 0
            assert N * p.L[i] >= n                      # everything fits
            if p.L[i] > 0:
                assert N * (p.L[i] - align) < n         # and no smaller multiple of align would
            else:
                assert n == 0
            assert sum(p.real_count(i, r) for r in range(N)) == n
            # padding sits at the tail: real counts are non-increasing in r
            counts = [p.real_count(i, r) for r in range(N)]
            assert counts == sorted(counts, reverse=True)


def test_brute_force_element_ownership():
    """Every element j of a variable lands in exactly one (replica, slot): r = j // L, k = j % L."""
    for N, align, numel in [(3, 1, [10, 1, 0, 7]), (4, 4, [17, 64, 5]), (5, 8, [100, 3])]:
        p = make_plan(numel, N, align)
        for i, n in enumerate(numel):
            owners = {}
            for r in range(N):
                for k in range(p.L[i]):
                    j = r * p.L[i] + k
                    if j < n:
                        assert j not in owners
                        owners[j] = (r, k)
                        assert k < p.real_count(i, r)
                    else:
                        assert k >= p.real_count(i, r)
            assert sorted(owners) == list(range(n))


def test_aux_memory_per_replica_is_V_over_N_plus_pad():
    # Section 4.2 (Memory saving): auxiliary bytes per replica shrink from V to V/N (+ padding).
    numel = [1000 * 128, 512 * 512, 512, 2048 * 512, 512 * 2048, 128]
    for N in (1, 2, 4, 8, 64):
        p = make_plan(numel, N, 8)
        assert p.S >= sum(numel) / N
        assert p.S - sum(numel) / N < 8 * len(numel)


def test_bad_arguments():
    with pytest.raises(ValueError):
        make_plan([4], 0)
    with pytest.raises(ValueError):
        make_plan([4], 2, 3)
    with pytest.raises(ValueError):
        make_plan([-1], 2)
