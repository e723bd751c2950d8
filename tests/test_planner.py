"""The planner entry points of the library (include/jupiter_plan.h, host code only) against the planner
oracle: the optimum values are unique and must agree; a reported partition is checked for validity and for
attaining the optimum (several partitions can be equally good)."""
import ctypes
import math
import random

import pytest

from oracle import planner as op
from paper_2504_08242_amd import binding as jb
from paper_2504_08242_amd import planner as jp

INF = math.inf


def random_table(rng, nx, ny, x_max, y_max):
    xs = sorted(rng.sample(range(1, x_max + 1), nx))
    ys = [0] + sorted(rng.sample(range(1, y_max + 1), ny - 1))
    # latency grows with both lengths, with noise: not convex, not separable
    q = [[0.2 + 0.01 * x * (1 + 0.002 * y) + rng.random() * 0.3 for y in ys] for x in xs]
    return xs, ys, q


def test_interpolated_q_equals_the_oracle_rule():
    rng = random.Random(5)
    xs, ys, q = random_table(rng, 6, 5, 300, 1000)
    plan = jp.SeqPlan(xs, ys, q, b=1, n_devices=1, s_max=400)
    for x in list(range(1, 400, 7)) + xs + [5000]:
        for y in [0, 1, 17, 250, 999, 1000, 1001, 4000] + ys:
            assert plan.q(x, y) == pytest.approx(op.interp_q(xs, ys, q, x, y), rel=1e-13, abs=1e-13), (x, y)
    assert math.isnan(plan.q(0, 0)) and math.isnan(plan.q(3, -1))


def test_q_stays_positive_outside_the_profiled_grid():
    """A y grid that does not start at 0: the first column is held below it (continued it would be -1 ms at y = 0),
    and no continued value falls below the smallest profiled latency."""
    plan = jp.SeqPlan([64, 128], [512, 1024], [[1.0, 3.0], [2.0, 6.0]], b=1, n_devices=2, s_max=1500)
    assert plan.q(64, 0) == 1.0 and plan.q(128, 100) == 2.0 and plan.q(96, 512) == 1.5
    assert plan.q(64, 768) == 2.0 and plan.q(64, 2048) == 7.0           # inside, and continued upwards
    falling = jp.SeqPlan([10, 20], [0, 100], [[5.0, 3.0], [2.0, 1.5]], b=1, n_devices=1, s_max=64)
    assert falling.q(40, 0) == 1.5 and falling.q(10, 1000) == 1.5        # floored at the smallest table entry
    for y in range(1, 1500, 37):
        for k in (1, 2, 3):
            lens, w, total = plan.partition(y, k) if y >= k else ([], 1.0, 1.0)
            assert w > 0 and total > 0


@pytest.mark.parametrize("b", [1, 3, 8])
def test_sequence_tables_equal_the_oracle_for_every_length_and_count(b):
    rng = random.Random(6 + b)
    xs, ys, q = random_table(rng, 5, 4, 40, 60)
    D, S = 2, 48
    plan = jp.SeqPlan(xs, ys, q, b=b, n_devices=D, s_max=S)
    qf = lambda x, l: op.interp_q(xs, ys, q, x, l)
    dp = op.SequenceDP(qf, b)
    for y in range(1, S + 1):
        for k in range(1, 4 * D + 1):
            want, _ = dp.W(y, k)
            if want == INF:
                with pytest.raises(jb.JupiterError) as ei:
                    plan.partition(y, k)
                assert ei.value.status == jb.JUP_ECAP
                continue
            lens, w, total = plan.partition(y, k)
            assert w == pytest.approx(want, rel=1e-12), (y, k)
            assert len(lens) == k and sum(lens) == y and min(lens) >= b
            h = op.chunk_latencies(qf, lens)
            assert max(h) == pytest.approx(w, rel=1e-12)            # the reported partition attains W
            assert total == pytest.approx(sum(h), rel=1e-12)        # and its latencies are summed for Eq. 4
        kb, lb, lat = op.choose_k(qf, y, b, D)
        if kb is None:
            with pytest.raises(jb.JupiterError) as ei:
                plan.best(y)
            assert ei.value.status == jb.JUP_ECAP
        else:
            k, lens, got = plan.best(y)
            assert got == pytest.approx(lat, rel=1e-12), y
            assert got == pytest.approx(op.pipeline_latency(qf, lens, D), rel=1e-12)
            assert len(lens) == k and sum(lens) == y


@pytest.mark.parametrize("granule", [2, 4, 7])
def test_aligned_sequence_tables_equal_the_oracle(granule):
    """jup_seq_plan_create_aligned: cut points on multiples of the granule, against the oracle's restricted recurrence
    and its enumeration; granule 1 is jup_seq_plan_create."""
    rng = random.Random(20 + granule)
    xs, ys, q = random_table(rng, 5, 4, 40, 60)
    D, S, b = 2, 40, 3
    plan = jp.SeqPlan(xs, ys, q, b=b, n_devices=D, s_max=S, granule=granule)
    plain = jp.SeqPlan(xs, ys, q, b=b, n_devices=D, s_max=S)
    one = jp.SeqPlan(xs, ys, q, b=b, n_devices=D, s_max=S, granule=1)
    qf = lambda x, l: op.interp_q(xs, ys, q, x, l)
    dp = op.SequenceDP(qf, b, granule)
    for y in range(1, S + 1):
        for k in range(1, 4 * D + 1):
            want, _ = dp.W(y, k)
            if want == INF:
                with pytest.raises(jb.JupiterError) as ei:
                    plan.partition(y, k)
                assert ei.value.status == jb.JUP_ECAP
            else:
                lens, w, total = plan.partition(y, k)
                assert w == pytest.approx(want, rel=1e-12), (y, k)
                assert len(lens) == k and sum(lens) == y and min(lens) >= b
                assert all(x % granule == 0 for x in lens[:-1]), lens
                assert max(op.chunk_latencies(qf, lens)) == pytest.approx(w, rel=1e-12)
                if y <= 16 and k <= 3:
                    assert w == pytest.approx(op.sequence_partition_bruteforce(qf, y, k, b, granule), rel=1e-12)
                assert w >= plain.partition(y, k)[1] * (1 - 1e-12)      # a restriction never helps
            try:
                assert one.partition(y, k) == plain.partition(y, k)
            except jb.JupiterError:
                pass
        kb, lb, lat = op.choose_k(qf, y, b, D, granule)
        if kb is not None:
            k, lens, got = plan.best(y)
            assert got == pytest.approx(lat, rel=1e-12), y
    with pytest.raises(jb.JupiterError) as ei:
        jp.SeqPlan(xs, ys, q, b=b, n_devices=D, s_max=S, granule=0)
    assert ei.value.status == jb.JUP_EINVAL


def test_sequence_partition_equals_enumeration_on_small_prompts():
    rng = random.Random(9)
    xs, ys, q = random_table(rng, 4, 3, 12, 12)
    plan = jp.SeqPlan(xs, ys, q, b=2, n_devices=1, s_max=12)
    qf = lambda x, l: op.interp_q(xs, ys, q, x, l)
    for y in range(2, 13):
        for k in range(1, 5):
            bf = op.sequence_partition_bruteforce(qf, y, k, 2)
            if bf == INF:
                continue
            assert plan.partition(y, k)[1] == pytest.approx(bf, rel=1e-12)


def test_measured_shape_later_sub_sequences_are_shorter_and_splitting_pays_on_several_stages():
    """A table of the shape measured on the MI355X stage: a floor for short chunks, then linear in x, plus a
    term in x*y for the attention over the prefix."""
    xs, ys = [16, 64, 128, 256, 512, 1024, 2048], [0, 512, 1024, 2048]
    q = [[max(0.9, 0.004 * x) + 2e-7 * x * (y + x / 2) for y in ys] for x in xs]
    plan = jp.SeqPlan(xs, ys, q, b=128, n_devices=4, s_max=2048)
    k, lens, lat = plan.best(2048)
    assert k >= 4 and all(a >= b for a, b in zip(lens, lens[1:])) and min(lens) >= 128
    assert lat < 4 * plan.q(2048, 0)                       # beats sending the whole prompt stage by stage
    assert plan.best(130)[0] == 1                           # too short to split into pieces of 128
    one = jp.SeqPlan(xs, ys, q, b=128, n_devices=1, s_max=2048)
    assert one.best(2048)[0] <= 2                           # one stage: nothing to overlap


def test_layer_partition_equals_the_oracle():
    rng = random.Random(7)
    assert jp.plan_layers([list(range(1, 10))] * 3, [0] * 9, [1] * 3) == ([5, 7, 9], 17.0)
    for _ in range(300):
        L, n = rng.randint(1, 12), rng.randint(1, 5)
        t = [[rng.choice([0.5, 1, 2, 3, 7]) for _ in range(L)] for _ in range(n)]
        mem = [rng.randint(1, 4) for _ in range(L)]
        budget = [rng.randint(3, 16) for _ in range(n)]
        want, cuts = op.layer_partition_dp(t, mem, budget)
        if want == INF:
            with pytest.raises(jb.JupiterError) as ei:
                jp.plan_layers(t, mem, budget)
            assert ei.value.status == jb.JUP_ECAP
            continue
        last, slowest = jp.plan_layers(t, mem, budget)
        assert slowest == want                                # sums of multiples of 0.5: exact
        assert last[-1] == L and all(a < b for a, b in zip(last, last[1:]))
        start, worst = 1, 0
        for dev, end in enumerate(last):
            worst = max(worst, op.stage_time(t, mem, budget, dev, start, end))
            start = end + 1
        assert worst == want


def test_planner_argument_errors():
    L = jp._lib()
    d3 = (ctypes.c_double * 3)(1, 1, 1)
    i3 = (ctypes.c_int32 * 3)()
    out = ctypes.c_double()
    assert L.jup_plan_layers(0, 1, d3, d3, d3, i3, ctypes.byref(out)) == jb.JUP_EINVAL
    assert L.jup_plan_layers(3, 1, None, d3, d3, i3, ctypes.byref(out)) == jb.JUP_EINVAL
    neg = (ctypes.c_double * 3)(1, -1, 1)
    assert L.jup_plan_layers(3, 1, neg, d3, d3, i3, ctypes.byref(out)) == jb.JUP_EINVAL
    assert L.jup_plan_layers(2, 3, (ctypes.c_double * 6)(*[1] * 6), d3, d3, i3, ctypes.byref(out)) == jb.JUP_ECAP
    with pytest.raises(jb.JupiterError):
        jp.SeqPlan([4, 4], [0], [[1.0], [2.0]], 1, 1, 8)         # xs not increasing
    with pytest.raises(jb.JupiterError):
        jp.SeqPlan([4, 8], [0], [[1.0], [0.0]], 1, 1, 8)         # a latency of zero
    with pytest.raises(jb.JupiterError):
        jp.SeqPlan([4, 8], [0], [[1.0], [2.0]], 0, 1, 8)         # b = 0
    plan = jp.SeqPlan([4, 8], [0, 8], [[1.0, 1.5], [2.0, 3.0]], 2, 2, 16)
    for y, k in ((0, 1), (17, 1), (8, 0), (8, 9)):
        with pytest.raises(jb.JupiterError) as ei:
            plan.partition(y, k)
        assert ei.value.status == jb.JUP_EINVAL
    with pytest.raises(jb.JupiterError) as ei:
        plan.best(1)
    assert ei.value.status == jb.JUP_ECAP
    assert L.jup_seq_plan_partition(None, 1, 1, None, None, None) == jb.JUP_EINVAL
    L.jup_seq_plan_destroy(None)
