"""Pins of the buffer-plan oracle (oracle/plan_oracle.py) against what the paper's definitions
fix by themselves: hand-worked programs, brute-force interference and optimality checks on random
programs, and a planted mistake that the checks must catch.  CPU only.

Sec. "Phase 4: IR Analysis & Optimization": Eq. "liveness", Alg. "Linear-Scan Buffer
Allocation", Eq. "buf_reduction".
"""
import random

import pytest

from oracle import plan_oracle as P


def random_program(rng, n_instr, fan_in=3, p_scratch=0.3, p_no_out=0.1):
    """SSA program: instruction j writes a fresh register and reads up to `fan_in` earlier ones;
    now and then it also mentions a scratch register nobody else touches, or has no output."""
    prog, n = [], 0
    for j in range(n_instr):
        ins = rng.sample(range(n), min(n, rng.randint(0, fan_in))) if n else []
        out = -1
        if rng.random() >= p_no_out or n == 0:
            out = n
            n += 1
        if rng.random() < p_scratch:
            ins = ins + [n]
            n += 1
        prog.append((out, ins))
    return prog, n


def overlaps(a, b):
    return not (a[1] < b[0] or b[1] < a[0])       # closed intervals intersect


def max_alive(intervals):
    ivs = [iv for iv in intervals if iv is not None]
    if not ivs:
        return 0
    last = max(e for _, e in ivs)
    return max(sum(1 for s, e in ivs if s <= t <= e) for t in range(last + 1))


# ------------------------------------------------------------------ hand-worked programs

def test_chain_alternates_two_buffers():
    # r0 = f(); r1 = f(r0); r2 = f(r1); ...: r_j lives [j, j+1].  r_{j+2} starts at j+2, strictly
    # after r_j ended (j+1), so it takes r_j's buffer; r_{j+1} is still read at j+2.
    n = 7
    prog = [(0, [])] + [(j, [j - 1]) for j in range(1, n)]
    iv = P.live_intervals(prog, n)
    assert iv == [(j, j + 1) for j in range(n - 1)] + [(n - 1, n - 1)]
    buf, m = P.linear_scan(iv)
    assert m == 2
    assert buf == [j % 2 for j in range(n)]
    assert P.buffer_reduction(m, n) == pytest.approx(1 - 2 / 7)


def test_diamond():
    # 0: a = in; 1: b = f(a); 2: c = g(a); 3: d = h(b, c)
    prog = [(0, []), (1, [0]), (2, [0]), (3, [1, 2])]
    iv = P.live_intervals(prog, 4)
    assert iv == [(0, 2), (1, 3), (2, 3), (3, 3)]
    buf, m = P.linear_scan(iv)
    # a, b, c are alive together at index 2; d starts at 3 when only a (ended at 2) is free
    assert (buf, m) == ([0, 1, 2, 0], 3)
    assert P.dead_after(iv) == {2: [0], 3: [1, 2, 3]}


def test_fan_out_keeps_the_source_alive():
    # a is read by the last instruction: nothing may reuse its buffer in between
    prog = [(0, []), (1, [0]), (2, [1]), (3, [2]), (4, [3, 0])]
    iv = P.live_intervals(prog, 5)
    assert iv[0] == (0, 4)
    buf, m = P.linear_scan(iv)
    assert all(buf[r] != buf[0] for r in range(1, 5))
    assert m == 3                                    # a, plus the alternating pair of the chain


def test_lowest_numbered_free_buffer_is_taken():
    # three registers die one after the other (ends 1, 2, 3); each of the three born at 5, 6 and
    # 7 lives for one instruction, so every one of them finds buffer 0 free again
    iv = [(0, 1), (0, 2), (0, 3), (5, 5), (6, 6), (7, 7)]
    buf, m = P.linear_scan(iv)
    assert m == 3
    assert buf == [0, 1, 2, 0, 0, 0]
    # buffers 2 and 3 come free together at index 2 (r4 takes 2, 3 stays free), buffer 1 at
    # index 4: r5 then has {1, 3} to choose from and takes the lower number, not the one that
    # has been free for longer
    iv = [(0, 9), (0, 3), (0, 1), (0, 1), (2, 9), (4, 9)]
    buf, m = P.linear_scan(iv)
    assert (buf, m) == ([0, 1, 2, 3, 2, 1], 4)


def test_scratch_register_and_unread_output():
    # r1 is a scratch area instruction 1 uses for itself (nobody writes it), r2 is never read
    prog = [(0, []), (2, [0, 1]), (-1, [0])]
    iv = P.live_intervals(prog, 4)
    assert iv == [(0, 2), (1, 1), (1, 1), None]
    buf, m = P.linear_scan(iv)
    assert buf[3] == -1 and m == 3


def test_equal_starts_go_by_register_number():
    iv = [(0, 0), (2, 4), (2, 3), (2, 2)]
    buf, m = P.linear_scan(iv)
    assert buf == [0, 0, 1, 2] and m == 3


# ------------------------------------------------------------------ properties, by brute force

@pytest.mark.parametrize("seed", range(40))
def test_random_programs_no_interference_and_optimal_count(seed):
    rng = random.Random(1000 + seed)
    prog, n = random_program(rng, rng.randint(1, 60), fan_in=rng.randint(1, 4))
    iv = P.live_intervals(prog, n)
    # Eq. "liveness", re-derived the slow way: scan every instruction for every register
    for r in range(n):
        where = [j for j, (out, ins) in enumerate(prog) if out == r or r in ins]
        assert iv[r] == ((where[0], where[-1]) if where else None)
    buf, m = P.linear_scan(iv)
    live = [r for r in range(n) if iv[r] is not None]
    for a in live:
        for b in live:
            if a < b and buf[a] == buf[b]:
                assert not overlaps(iv[a], iv[b]), (a, b, iv[a], iv[b])
    assert sorted(set(buf[r] for r in live)) == list(range(m))
    assert m == max_alive(iv)
    # dead-after: every live register exactly once, at its end
    dead = P.dead_after(iv)
    seen = sorted(r for regs in dead.values() for r in regs)
    assert seen == live
    for j, regs in dead.items():
        assert all(iv[r][1] == j for r in regs)
    if live:
        assert P.buffer_reduction(m, len(live)) == pytest.approx(1 - m / len(live))


def test_a_wrong_expiry_test_is_caught():
    # the same scan with "ended at or before the start" lets an instruction's output share the
    # buffer of one of its inputs; the interference check above must reject that plan
    def scan_wrong(intervals):
        order = sorted(range(len(intervals)), key=lambda r: (intervals[r][0], r))
        buf, active, pool, nb = [-1] * len(intervals), [], [], 0
        for r in order:
            s, e = intervals[r]
            keep = []
            for (ej, bj) in active:
                (pool if ej <= s else keep).append(bj if ej <= s else (ej, bj))
            active = keep
            if pool:
                b = pool.pop(0)
            else:
                b, nb = nb, nb + 1
            buf[r] = b
            active.append((e, b))
        return buf, nb

    prog = [(0, [])] + [(j, [j - 1]) for j in range(1, 6)]
    iv = P.live_intervals(prog, 6)
    bad, _ = scan_wrong(iv)
    clash = [(a, b) for a in range(6) for b in range(a + 1, 6)
             if bad[a] == bad[b] and overlaps(iv[a], iv[b])]
    assert clash, "the planted mistake must produce an interference"
    good, _ = P.linear_scan(iv)
    assert not [(a, b) for a in range(6) for b in range(a + 1, 6)
                if good[a] == good[b] and overlaps(iv[a], iv[b])]


# ------------------------------------------------------------------ byte plan

@pytest.mark.parametrize("seed", range(20))
def test_workspace_plan_regions_of_live_registers_never_overlap(seed):
    rng = random.Random(7000 + seed)
    prog, n = random_program(rng, rng.randint(2, 50))
    iv = P.live_intervals(prog, n)
    sizes = [rng.choice([100, 256, 4096, 5000, 65536]) for _ in range(n)]
    off, total, nb = P.workspace_plan(iv, sizes)
    live = [r for r in range(n) if iv[r] is not None]
    for r in live:
        assert off[r] % 256 == 0 and off[r] + sizes[r] <= total
    for a in live:
        for b in live:
            if a < b and overlaps(iv[a], iv[b]):
                assert off[a] + sizes[a] <= off[b] or off[b] + sizes[b] <= off[a], (a, b)
    # each group is an independent linear scan: its buffer count is its own max overlap; the
    # registers living within one instruction form one group sized to the largest of them
    single = [r for r in live if iv[r][0] == iv[r][1]]
    multi = [r for r in live if iv[r][0] != iv[r][1]]
    pad = lambda b: (b + 255) // 256 * 256
    expect_bufs = max_alive([iv[r] for r in single])
    expect_total = pad(max([sizes[r] for r in single] or [0])) * expect_bufs
    for size in set(sizes[r] for r in multi):
        k = max_alive([iv[r] for r in multi if sizes[r] == size])
        expect_bufs += k
        expect_total += pad(size) * k
    assert nb == expect_bufs
    assert total == expect_total


def test_workspace_plan_hand_worked():
    # r0 [0,2] 1000 B, r1 [1,1] 64 B (scratch), r2 [2,3] 1000 B, r3 [3,3] 4096 B (scratch), r4 [3,4] 1000 B
    iv = [(0, 2), (1, 1), (2, 3), (3, 3), (3, 4)]
    off, total, nb = P.workspace_plan(iv, [1000, 64, 1000, 4096, 1000])
    # group "1000 B": r0 -> buffer 0, r2 overlaps r0 at index 2 -> buffer 1, r4 starts at 3 after r0
    # ended at 2 -> buffer 0; stride 1024.  group "single": one buffer of 4096 B after it.
    assert off == [0, 2048, 1024, 2048, 0]
    assert (total, nb) == (2048 + 4096, 3)
