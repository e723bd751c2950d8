"""Pins of the planner oracle (oracle/planner.py): the two dynamic programs of Sec. IV-B against exhaustive
enumeration, textbook instances, closed forms and hand-worked examples; the interpolation of q(x, y) against
functions a bilinear rule reproduces exactly."""
import itertools
import math
import random

import numpy as np
import pytest

from oracle import planner as op

INF = math.inf


# ---- Eq. 1 ------------------------------------------------------------------------------------------
def test_layer_partition_textbook_instance():
    """The linear-partition example of Skiena's Algorithm Design Manual: 1..9 into 3 ranges -> 1-5 | 6-7 | 8-9, max 17."""
    t = [list(range(1, 10))] * 3
    best, cuts = op.layer_partition_dp(t, [0] * 9, [1] * 3)
    assert best == 17 and cuts == (5, 7, 9)
    best, cuts = op.layer_partition_dp([[1] * 9] * 3, [0] * 9, [1] * 3)
    assert best == 3 and cuts == (3, 6, 9)


def test_layer_partition_closed_forms():
    for L, n in ((10, 3), (7, 7), (12, 5), (5, 1)):
        best, cuts = op.layer_partition_dp([[2.5] * L] * n, [1] * L, [L] * n)
        assert best == 2.5 * math.ceil(L / n)
        assert len(cuts) == n and cuts[-1] == L and all(a < b for a, b in zip(cuts, cuts[1:]))
    # fewer layers than devices: no partition gives every device a layer
    assert op.layer_partition_dp([[1.0] * 2] * 3, [1] * 2, [9] * 3)[0] == INF


def test_layer_partition_heterogeneous_devices_and_memory_budget():
    # the second device is twice as slow: 4 + 2 layers balance at 4
    best, cuts = op.layer_partition_dp([[1] * 6, [2] * 6], [1] * 6, [6, 6])
    assert best == 4 and cuts == (4, 6)
    # ... unless the fast device only has room for 3 layers: then 3 | 3 at cost 6
    best, cuts = op.layer_partition_dp([[1] * 6, [2] * 6], [1] * 6, [3, 6])
    assert best == 6 and cuts == (3, 6)
    # ... and with room for 3 + 2 nothing fits
    assert op.layer_partition_dp([[1] * 6, [2] * 6], [1] * 6, [3, 2])[0] == INF
    # the order of the devices matters: the slow one first takes the first layers
    best, cuts = op.layer_partition_dp([[2] * 6, [1] * 6], [1] * 6, [6, 6])
    assert best == 4 and cuts == (2, 6)


def test_layer_partition_dp_equals_enumeration():
    rng = random.Random(1)
    for _ in range(200):
        L, n = rng.randint(1, 9), rng.randint(1, 4)
        t = [[rng.choice([0.5, 1, 2, 3, 7]) for _ in range(L)] for _ in range(n)]
        mem = [rng.randint(1, 4) for _ in range(L)]
        budget = [rng.randint(3, 14) for _ in range(n)]
        dp, cuts = op.layer_partition_dp(t, mem, budget)
        bf = op.layer_partition_bruteforce(t, mem, budget) if L >= n else INF
        assert dp == bf, (t, mem, budget)
        if dp < INF:  # the reported cuts realise the optimum
            start, worst = 1, 0
            for dev, end in enumerate(cuts):
                worst = max(worst, op.stage_time(t, mem, budget, dev, start, end))
                start = end + 1
            assert worst == dp and cuts[-1] == L


# ---- Eq. 2-4 ------------------------------------------------------------------------------------------
def test_sequence_partition_with_latency_proportional_to_length():
    """q(x, l) = x: the slowest of k pieces of y tokens is ceil(y / k), if every piece can have b tokens."""
    q = lambda x, l: float(x)
    for y, k, b in itertools.product((7, 12, 33), (1, 2, 3, 5), (1, 3, 6)):
        w, lens = op.sequence_partition_dp(q, y, k, b)
        if y < k * b:
            assert w == INF
        else:
            assert w == math.ceil(y / k), (y, k, b)
            assert sum(lens) == y and len(lens) == k and min(lens) >= b


def test_sequence_partition_hand_worked_example():
    """q(x, l) = x (l + x): 6 tokens in 2 pieces.  Splits (1,5)..(5,1) cost max(1, 5*6)=30, max(4, 4*6)=24,
    max(9, 3*6)=18, max(16, 2*6)=16, max(25, 1*6)=25: the best is (4, 2) at 16 -- the later piece is shorter."""
    q = lambda x, l: float(x * (l + x))
    assert op.sequence_partition_dp(q, 6, 2, 1) == (16.0, (4, 2))
    assert op.sequence_partition_dp(q, 6, 2, 3) == (18.0, (3, 3))     # b = 3 leaves one split
    assert op.sequence_partition_dp(q, 6, 1, 1) == (36.0, (6,))
    # Eq. 4 on 3 devices: (4, 2) -> 16 + 12 + 2 * 16 = 60; one piece -> 36 + 2 * 36 = 108
    assert op.pipeline_latency(q, (4, 2), 3) == 60.0
    assert op.pipeline_latency(q, (6,), 3) == 108.0


def test_later_sub_sequences_are_not_longer_when_the_prefix_costs():
    """Fig. 7 (left): with attention over the prefix, a balanced partition shortens the later pieces."""
    q = lambda x, l: x * (100.0 + l + 0.5 * x)
    for y, k in ((64, 4), (100, 3), (90, 6)):
        w, lens = op.sequence_partition_dp(q, y, k, 1)
        assert all(a >= b for a, b in zip(lens, lens[1:])), lens
        assert lens[0] > lens[-1]
        assert w == max(op.chunk_latencies(q, lens))


def test_sequence_partition_dp_equals_enumeration():
    rng = random.Random(2)
    for trial in range(30):
        tab = {(x, l): rng.choice([1.0, 2.0, 3.5, 5.0, 8.0]) + 0.25 * x + 0.1 * l for x in range(1, 14) for l in range(14)}
        q = lambda x, l: tab[(x, l)]
        for y in range(1, 13):
            for k in range(1, 5):
                for b in (1, 2, 3):
                    w, lens = op.sequence_partition_dp(q, y, k, b)
                    assert w == op.sequence_partition_bruteforce(q, y, k, b), (trial, y, k, b)
                    if w < INF:
                        assert sum(lens) == y and len(lens) == k and min(lens) >= b
                        assert max(op.chunk_latencies(q, lens)) == w


def test_sequence_partition_with_aligned_cut_points():
    """granule g: every sub-sequence but the last is a multiple of g.  DP == enumeration over exactly those
    partitions; granule 1 is the unrestricted recurrence; a closed form: latency proportional to length, y = 4 g + 1
    into 2 pieces: the cut is at 2 g (pieces 2 g and 2 g + 1), at 3 pieces at g and 2 g... the best of the aligned ones."""
    rng = random.Random(5)
    for trial in range(10):
        tab = {(x, l): rng.choice([1.0, 2.0, 3.5, 5.0]) + 0.25 * x + 0.1 * l for x in range(1, 26) for l in range(26)}
        q = lambda x, l: tab[(x, l)]
        for g in (1, 2, 4, 5):
            for y in range(1, 25):
                for k in range(1, 5):
                    for b in (1, 3):
                        w, lens = op.sequence_partition_dp(q, y, k, b, g)
                        assert w == op.sequence_partition_bruteforce(q, y, k, b, g), (trial, g, y, k, b)
                        if w < INF:
                            assert sum(lens) == y and len(lens) == k and min(lens) >= b
                            assert all(x % g == 0 for x in lens[:-1]), (g, lens)
                            assert max(op.chunk_latencies(q, lens)) == w
                        if g == 1:
                            assert (w, lens) == op.sequence_partition_dp(q, y, k, b)
    q = lambda x, l: float(x)
    assert op.sequence_partition_dp(q, 4 * 8 + 1, 2, 1, 8) == (17.0, (16, 17))
    assert op.sequence_partition_dp(q, 4 * 8 + 1, 2, 1, 1) == (17.0, (16, 17))
    assert op.sequence_partition_dp(q, 33, 3, 1, 8) == (16.0, (8, 16, 9))        # aligned: no better than a piece of 16
    assert op.sequence_partition_dp(q, 33, 3, 1, 1)[0] == 11.0                   # unrestricted: 11 + 11 + 11
    assert op.sequence_partition_dp(q, 7, 2, 1, 8) == (INF, None)                # no multiple of 8 below 7
    assert op.choose_k(lambda x, l: 6.0 + x, 48, 1, 4, 16)[1] == (16, 16, 16)   # three aligned pieces beat 2 and 1


def test_choice_of_k_minimises_the_latency_estimate():
    """Eq. 4 by hand: per-chunk overhead c, work proportional to length: Latency(k) = kc + y + (D-1)(c + y/k)."""
    c, y, D = 6.0, 48, 4
    q = lambda x, l: c + x
    k, lens, lat = op.choose_k(q, y, 1, D)
    want = {kk: kk * c + y + (D - 1) * (c + math.ceil(y / kk)) for kk in range(1, 4 * D + 1)}
    assert lat == min(want.values()) and want[k] == lat
    assert k == 4 and lens == (12, 12, 12, 12)      # 24 + 48 + 3 * 18 = 126; k = 3: 18 + 48 + 66 = 132; k = 6: 36 + 48 + 42 = 126
    # one device: nothing to overlap, splitting only adds overhead
    assert op.choose_k(q, y, 1, 1)[0] == 1
    # a minimum length of 16 leaves k <= 3
    assert op.choose_k(q, y, 16, D)[0] == 3


# ---- q(x, y) between profiled points ---------------------------------------------------------------------
def test_interpolation_reproduces_the_table_and_bilinear_functions():
    xs, ys = [16, 64, 256, 512], [0, 512, 2048]
    f = lambda x, y: 3.0 + 0.5 * x + 0.01 * y + 0.002 * x * y       # bilinear: reproduced exactly inside the grid
    tab = [[f(x, y) for y in ys] for x in xs]
    for i, x in enumerate(xs):
        for j, y in enumerate(ys):
            assert op.interp_q(xs, ys, tab, x, y) == tab[i][j]
    for x, y in ((16, 0), (40, 100), (64, 511), (300, 2048), (512, 1000), (100, 0)):
        assert op.interp_q(xs, ys, tab, x, y) == pytest.approx(f(x, y), rel=1e-12)
    # midpoint of a cell = mean of its corners
    assert op.interp_q(xs, ys, tab, 40, 256) == pytest.approx((tab[0][0] + tab[0][1] + tab[1][0] + tab[1][1]) / 4)
    # continued linearly above the largest x and above the largest y
    assert op.interp_q(xs, ys, tab, 768, 0) == pytest.approx(f(768, 0), rel=1e-12)
    assert op.interp_q(xs, ys, tab, 64, 4096) == pytest.approx(f(64, 4096), rel=1e-12)
    # below the smallest profiled chunk the latency stays that of the smallest
    assert op.interp_q(xs, ys, tab, 5, 512) == tab[0][1]
    # agrees with numpy's 1-D rule along each axis
    col = [row[1] for row in tab]
    assert op.interp_q(xs, ys, tab, 200, 512) == pytest.approx(np.interp(200, xs, col), rel=1e-12)
    assert op.interp_q(xs, ys, tab, 256, 1234) == pytest.approx(np.interp(1234, ys, tab[2]), rel=1e-12)
    # below the smallest profiled prefix the latency of that prefix is held: continued downwards the segment
    # {512: 1 ms, 1024: 3 ms} would give -1 ms at y = 0, and Eq. 2-4 mean nothing for such a latency
    assert op.interp_q([64], [512, 1024], [[1.0, 3.0]], 64, 0) == 1.0
    assert op.interp_q([64], [512, 1024], [[1.0, 3.0]], 64, 768) == 2.0
    assert op.interp_q([64], [512, 1024], [[1.0, 3.0]], 64, 2048) == 7.0
    # a falling outermost segment continued upwards stops at the smallest profiled latency instead of crossing zero
    assert op.interp_q([64], [0, 100], [[3.0, 1.0]], 64, 150) == 1.0
    assert op.interp_q([10, 20], [0], [[5.0], [2.0]], 40, 0) == 2.0
    # a single profiled column or row
    assert op.interp_q([64], [0, 100], [[1.0, 3.0]], 500, 50) == 2.0
    assert op.interp_q([64, 128], [0], [[1.0], [3.0]], 96, 700) == 2.0
