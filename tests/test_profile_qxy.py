"""The q(x, y) profiler (Sec. IV-B.2) and the way its table reaches the planner: table, knee and CSV logic on the CPU;
one small measurement on the GPU."""
import os

import numpy as np
import pytest

from paper_2504_08242_amd import planner, profile_qxy

PKG = os.path.dirname(os.path.abspath(profile_qxy.__file__))
SHIPPED = os.path.join(PKG, "qxy_mi355x_7b_stage.csv")


def synthetic_table(xs, ys):
    # a stage that costs 0.8 ms for its weights, 2.5 us per token and 0.05 us per (token, 1024 cached) pair
    return {(x, y): 0.8 + 2.5e-3 * x + 5e-8 * x * y for x in xs for y in ys}


def test_knee_is_the_smallest_chunk_within_20_percent_of_the_best_rate():
    xs, ys = [16, 64, 256, 1024, 4096], [0, 1024]
    t = synthetic_table(xs, ys)
    rate = {x: x / t[(x, 0)] for x in xs}
    want = min(x for x in xs if rate[x] >= 0.8 * max(rate.values()))
    assert profile_qxy.knee(t, xs, 0) == want == 1024
    assert profile_qxy.knee(t, xs, 0, within=1.0) == 4096
    flat = {(x, 0): 1e-3 * x for x in xs}                      # perfectly linear: every chunk is as good as the best
    assert profile_qxy.knee(flat, xs, 0) == 16


def test_table_text_has_one_row_per_x_and_one_column_per_y():
    xs, ys = [16, 128, 512], [0, 512, 2048]
    text = profile_qxy.format_table(synthetic_table(xs, ys), xs, ys, "title line")
    lines = text.splitlines()
    assert lines[0] == "title line" and len(lines) == 2 + len(xs) + 1
    for x, line in zip(xs, lines[2:]):
        cells = line.split()
        assert int(cells[0]) == x and len(cells) == 1 + len(ys) + 1
        assert float(cells[1]) == pytest.approx(0.8 + 2.5e-3 * x, abs=5e-4)
    assert "b = " in lines[-1]


def test_csv_round_trip_into_the_planner(tmp_path):
    xs, ys = [32, 128, 512, 2048], [0, 1024, 4096]
    t = synthetic_table(xs, ys)
    path = str(tmp_path / "q.csv")
    profile_qxy.write_csv(t, path)
    rx, ry, q = planner.read_qxy_csv(path)
    assert rx == xs and ry == ys
    assert np.allclose(q, [[t[(x, y)] for y in ys] for x in xs], atol=1e-4)
    plan = planner.SeqPlan(rx, ry, q, b=64, n_devices=4, s_max=2048)
    assert plan.q(128, 1024) == pytest.approx(t[(128, 1024)], abs=1e-4)       # a grid point comes back as written
    k, lens, lat = plan.best(1500)
    assert sum(lens) == 1500 and len(lens) == k and min(lens) >= 64 and lat > 0


def test_shipped_table_feeds_the_planner_and_is_monotone():
    """The table measured on the MI355X that ships as the planner's default."""
    xs, ys, q = planner.read_qxy_csv(SHIPPED)
    q = np.asarray(q)
    assert q.shape == (len(xs), len(ys)) and (q > 0).all()
    assert (np.diff(q, axis=1) > 0).all(), "a longer cached prefix never makes a chunk cheaper"
    assert (np.diff(q[xs.index(64):], axis=0) > 0).all(), "from 64 tokens on a longer chunk costs more"
    plan = planner.SeqPlan(xs, ys, q.tolist(), b=256, n_devices=4, s_max=2048)
    for y in (260, 1024, 2048):
        k, lens, lat = plan.best(y)
        assert sum(lens) == y and len(lens) == k and (k == 1 or min(lens) >= 256)
        parts, w, total = plan.partition(y, k)
        assert parts == lens and lat == pytest.approx(total + 3 * w, rel=1e-12)   # Eq. 4 with |D| = 4


@pytest.mark.gpu
def test_measured_q_grows_with_the_prefix_and_feeds_the_planner(tmp_path):
    from paper_2504_08242_amd import synth_inputs as si
    cfg = dict(si.LLAMA7B_STAGE, n_layers=1)
    xs, ys = [64, 256], [0, 2048, 8192]
    t = profile_qxy.measure(cfg, xs, ys, reps=10)
    assert set(t) == {(x, y) for x in xs for y in ys} and all(v > 0 for v in t.values())
    for x in xs:   # 8192 cached positions against none: far above timer noise (y = 2048 lies in between, not asserted)
        assert t[(x, 8192)] > t[(x, 0)], (x, t)
    assert t[(256, 8192)] > t[(64, 8192)] and t[(256, 0)] > 0.8 * t[(64, 0)]
    path = str(tmp_path / "q.csv")
    profile_qxy.write_csv(t, path)
    rx, ry, q = planner.read_qxy_csv(path)
    plan = planner.SeqPlan(rx, ry, q, b=64, n_devices=2, s_max=512)
    k, lens, lat = plan.best(512)
    assert sum(lens) == 512 and min(lens) >= 64 and lat > 0
    print(profile_qxy.format_table(t, xs, ys, "q(x,y) in ms, one 7B-shaped layer"), flush=True)
