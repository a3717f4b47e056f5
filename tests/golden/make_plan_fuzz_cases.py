#!/usr/bin/env python3
"""Writes tests/golden/plan_fuzz_cases.txt: seeded random and near-overflow inputs for the host-side plan and
replica-array arithmetic, with the values the CPU oracle gives for them (Python integers, no overflow).  Calls
only oracle/.  The sanitizer build of the library's host sources (tests/plan_fuzz.cpp) replays the file.

Line formats (fields separated by single spaces; lists by commas):
  plan <must|may> <N> <align> <chunk> <V> <n_0,...|-> <S> <total> <fold> <real_fold_r0> <real_fold_rlast>
  rows <must|may> <N> <align> <chunk> <V> <r_0xc_0,...|-> <S> <total> <fold> <real_fold_r0> <real_fold_rlast>
      must: the library has to accept the plan and agree; may: it may refuse (sizes beyond what a launch can
      address), but if it accepts it has to agree.  fold = sum_i (i+1) * (31 * L_i + off_i) mod (2^61 - 1);
      real_fold_r = sum_i (i+1) * real_count(i, r) mod (2^61 - 1).
  part <rows> <cols> <replica> <group> <shard_id> <two_phase_id> <first and last of shard_group> <first and last of reduce_group>
  cut <total> <parts> <part> <start> <length>
"""
import os
import random
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402

MOD = (1 << 61) - 1


def fold(plan):
    return sum((i + 1) * (31 * plan.L[i] + plan.off[i]) for i in range(plan.V)) % MOD


def real_fold(plan, r):
    return sum((i + 1) * plan.real_count(i, r) for i in range(plan.V)) % MOD


def cheap_or_refused(plan, N):
    """Keeps the replay fast: a case is either small enough to build in no time or so large that the library has
    to refuse it before building anything (more work items than a launch can hold)."""
    chunks = sum(-(-L // 2048) for L in plan.L)
    return chunks <= (1 << 16) or chunks * 2 * N > (1 << 33)


def main():
    rng = random.Random(20041336)
    out = []
    interesting = [0, 1, 2, 7, 8, 9, 63, 64, 65, 1023, 1024, 1025, 2047, 2048, 2049, 4095, 4097, 65535, 65537, 1000003]
    for case in range(160):
        N = rng.choice([1, 2, 3, 4, 7, 8, 10, 16, 31, 64, 130, 257, 1024, 2048])
        align = rng.choice([1, 2, 4, 8, 16, 64])
        chunk = rng.choice([0, 1024, 2048, 4096, 16384])
        V = rng.choice([0, 1, 2, 3, 5, 9, 17, 40])
        numel = [rng.choice(interesting) if rng.random() < 0.5 else rng.randrange(0, 300000) for _ in range(V)]
        p = oracle.make_plan(numel, N, align)
        out.append("plan must %d %d %d %d %s %d %d %d %d %d" % (
            N, align, chunk, V, ",".join(map(str, numel)) or "-", p.S, sum(numel), fold(p), real_fold(p, 0), real_fold(p, N - 1)))
    for case in range(80):
        N = rng.choice([1, 2, 3, 4, 8, 10, 16, 33, 64, 500])
        align = rng.choice([1, 2, 8, 32])
        chunk = rng.choice([0, 1024, 2048, 8192])
        V = rng.choice([0, 1, 2, 4, 9])
        shapes = [(rng.choice([0, 1, 2, 3, 9, 10, 64, 100, 513, 3001]), rng.choice([0, 1, 2, 7, 8, 64, 65, 256, 1000])) for _ in range(V)]
        p = oracle.make_row_plan(shapes, N, align)
        out.append("rows must %d %d %d %d %s %d %d %d %d %d" % (
            N, align, chunk, V, ",".join("%dx%d" % s for s in shapes) or "-", p.S, sum(a * b for a, b in shapes), fold(p),
            real_fold(p, 0), real_fold(p, N - 1)))
    # near the limits of 64-bit arithmetic: the library may refuse, it may not overflow
    huge = [(1 << 59), (1 << 59) - 1, (1 << 59) + 1, (1 << 62), (1 << 63) - 1, (1 << 45), (1 << 50) + 12345, (1 << 58) + 7]
    for case in range(90):
        N = rng.choice([1, 2, 8, 1024, 1 << 20, (1 << 31) - 1])
        align = rng.choice([1, 8, 1 << 20, 1 << 30])
        V = rng.choice([1, 2, 3, 17, 40])
        numel = [rng.choice(huge) if rng.random() < 0.7 else rng.randrange(0, 5000) for _ in range(V)]
        p = oracle.make_plan(numel, N, align)
        if not cheap_or_refused(p, N):
            continue
        out.append("plan may %d %d 0 %d %s %d %d %d %d %d" % (
            N, align, V, ",".join(map(str, numel)), p.S, sum(numel), fold(p), real_fold(p, 0), real_fold(p, N - 1)))
    # crafted: every piece passes the per-variable limits, only the running totals can overflow
    kmax = ((1 << 63) - 1) // 16
    for N in ((1 << 31) - 1, 1 << 30, 1 << 20):
        n = N * (kmax // N)
        for V in (15, 16, 17, 33):
            numel = [n] * V
            p = oracle.make_plan(numel, N, 1)
            out.append("plan may %d 1 0 %d %s %d %d %d %d %d" % (
                N, V, ",".join(map(str, numel)), p.S, sum(numel), fold(p), real_fold(p, 0), real_fold(p, N - 1)))
    for case in range(60):
        N = rng.choice([1, 3, 8, 1 << 20])
        V = rng.choice([1, 2, 5])
        shapes = [(rng.choice([(1 << 31), (1 << 40), (1 << 59), 3, 1000]), rng.choice([(1 << 31) + 1, (1 << 33), (1 << 59), 1, 64])) for _ in range(V)]
        p = oracle.make_row_plan(shapes, N, 8)
        if not cheap_or_refused(p, N):
            continue
        out.append("rows may %d 8 0 %d %s %d %d %d %d %d" % (
            N, V, ",".join("%dx%d" % s for s in shapes), p.S, sum(a * b for a, b in shapes), fold(p), real_fold(p, 0),
            real_fold(p, N - 1)))
    for case in range(80):
        rows = rng.choice([1, 2, 3, 8, 64, 1000])
        cols = rng.choice([1, 2, 4, 8, 32, 2048])
        replica = rng.randrange(rows * cols)
        group, sid, sg, rg = oracle.partial_sharding(rows, cols, replica)
        out.append("part %d %d %d %d %d %d %d %d %d %d" % (rows, cols, replica, group, sid,
                                                          oracle.two_phase_shard_id(rows, cols, replica), sg[0], sg[-1], rg[0], rg[-1]))
    for case in range(80):
        total = rng.choice([0, 1, 7, 4096, 1000003, (1 << 40) + 3, (1 << 62)])
        parts = rng.choice([1, 2, 3, 8, 1000, (1 << 31) - 1])
        part = rng.randrange(parts)
        start, length = oracle.concat_partition(total, parts, part)
        out.append("cut %d %d %d %d %d" % (total, parts, part, start, length))
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "plan_fuzz_cases.txt")
    with open(path, "w") as f:
        f.write("# written by tests/golden/make_plan_fuzz_cases.py from oracle/ (see its docstring for the format)\n")
        f.write("\n".join(out) + "\n")
    print(path, len(out), "cases")


if __name__ == "__main__":
    main()
