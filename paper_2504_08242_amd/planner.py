#!/usr/bin/env python3
"""Thin ctypes front end of the planner entry points (include/jupiter_plan.h), and a small command line.

The planner of the Jupiter paper (Sec. IV-B) decides, from profiled latencies, where to cut the model into
stages (Eq. 1) and every prompt into sub-sequences (Eq. 2-4).  All arithmetic runs in libjupiter_stage.so;
this module only marshals arguments.

    python -m paper_2504_08242_amd.profile_qxy --csv q.csv          # on the MI355X: measures q(x, y)
    python -m paper_2504_08242_amd.planner --qxy q.csv --devices 4 --b 128 --lengths 260 1024 2048
"""
import argparse
import csv
import ctypes
import os

from . import binding as jb

_i32, _f64, _vp = ctypes.c_int32, ctypes.c_double, ctypes.c_void_p
_ready = False


def _lib():
    global _ready
    L = jb.lib()
    if not _ready:
        pi, pd = ctypes.POINTER(_i32), ctypes.POINTER(_f64)
        sig = {
            "jup_plan_layers": (_i32, [_i32, _i32, pd, pd, pd, pi, pd]),
            "jup_seq_plan_create": (_i32, [pi, _i32, pi, _i32, pd, _i32, _i32, _i32, ctypes.POINTER(_vp)]),
            "jup_seq_plan_create_aligned": (_i32, [pi, _i32, pi, _i32, pd, _i32, _i32, _i32, _i32, ctypes.POINTER(_vp)]),
            "jup_seq_plan_destroy": (None, [_vp]),
            "jup_seq_plan_q": (_f64, [_vp, _i32, _i32]),
            "jup_seq_plan_partition": (_i32, [_vp, _i32, _i32, pi, pd, pd]),
            "jup_seq_plan_best": (_i32, [_vp, _i32, pi, pi, pd]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _ready = True
    return L


def _arr(ctype, values):
    values = list(values)
    return (ctype * max(1, len(values)))(*values)


def plan_layers(layer_time, layer_mem, mem_budget):
    """layer_time[n][l], layer_mem[l], mem_budget[n] -> (last layer of every stage (1-based), slowest stage time)."""
    n_dev, n_layers = len(layer_time), len(layer_mem)
    assert all(len(row) == n_layers for row in layer_time) and len(mem_budget) == n_dev
    flat = [float(v) for row in layer_time for v in row]
    last = (_i32 * max(1, n_dev))()
    slowest = _f64()
    jb._check(_lib().jup_plan_layers(n_layers, n_dev, _arr(_f64, flat), _arr(_f64, map(float, layer_mem)),
                                     _arr(_f64, map(float, mem_budget)), last, ctypes.byref(slowest)))
    return list(last)[:n_dev], slowest.value


class SeqPlan:
    """The solved sequence-partition tables for every prompt length up to s_max (Eq. 2-4)."""

    def __init__(self, xs, ys, q, b, n_devices, s_max, granule=1):
        """q[i][j]: profiled latency of a sub-sequence of xs[i] tokens behind ys[j] cached ones.  granule: cut points
        are multiples of it (jup_seq_plan_create_aligned; 1 = the paper's recurrence)."""
        assert len(q) == len(xs) and all(len(row) == len(ys) for row in q)
        self.n_devices, self.s_max, self.b, self.granule = int(n_devices), int(s_max), int(b), int(granule)
        self.handle = _vp()
        flat = [float(v) for row in q for v in row]
        jb._check(_lib().jup_seq_plan_create_aligned(_arr(_i32, map(int, xs)), len(xs), _arr(_i32, map(int, ys)), len(ys),
                                                     _arr(_f64, flat), self.b, self.granule, self.n_devices, self.s_max,
                                                     ctypes.byref(self.handle)))

    def q(self, x, y):
        return float(_lib().jup_seq_plan_q(self.handle, int(x), int(y)))

    def partition(self, y, k):
        """-> (lengths, slowest sub-sequence latency W(1..y, k), sum of the sub-sequence latencies)."""
        lengths = (_i32 * max(1, int(k)))()
        w, total = _f64(), _f64()
        jb._check(_lib().jup_seq_plan_partition(self.handle, int(y), int(k), lengths, ctypes.byref(w),
                                                ctypes.byref(total)))
        return list(lengths)[:k], w.value, total.value

    def best(self, y):
        """-> (k, lengths, estimated latency of Eq. 4)."""
        lengths = (_i32 * (4 * self.n_devices))()
        k, lat = _i32(), _f64()
        jb._check(_lib().jup_seq_plan_best(self.handle, int(y), ctypes.byref(k), lengths, ctypes.byref(lat)))
        return k.value, list(lengths)[:k.value], lat.value

    def destroy(self):
        if self.handle:
            _lib().jup_seq_plan_destroy(self.handle)
            self.handle = _vp()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def read_qxy_csv(path):
    """The x,y,ms file written by profile_qxy --csv -> (xs, ys, q[i][j])."""
    cells = {}
    with open(path) as f:
        for row in csv.DictReader(f):
            cells[(int(row["x"]), int(row["y"]))] = float(row["ms"])
    xs = sorted({x for x, _ in cells})
    ys = sorted({y for _, y in cells})
    return xs, ys, [[cells[(x, y)] for y in ys] for x in xs]


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--qxy", default=os.path.join(os.path.dirname(os.path.abspath(__file__)), "qxy_mi355x_7b_stage.csv"),
                    help="x,y,ms table of one stage (profile_qxy --csv); default: the table measured for the 8-layer "
                         "7B-shaped bf16 stage on one MI355X")
    ap.add_argument("--devices", type=int, default=4, help="stages of the pipeline, all as fast as the profiled one")
    ap.add_argument("--b", type=int, default=128, help="shortest sub-sequence that keeps the device busy")
    ap.add_argument("--lengths", type=int, nargs="+", default=[260, 512, 1024, 2048])
    ap.add_argument("--granule", type=int, default=1,
                    help="cut points are multiples of this many tokens (1: the paper's recurrence; 256: the row tile of "
                         "this GPU's kernels, where a coarse q(x, y) table is true)")
    args = ap.parse_args()
    xs, ys, q = read_qxy_csv(args.qxy)
    plan = SeqPlan(xs, ys, q, args.b, args.devices, max(args.lengths), granule=args.granule)
    for y in args.lengths:
        k, lens, lat = plan.best(y)
        one = plan.q(y, 0) * args.devices   # no intra-sequence pipelining: the prompt crosses the stages one by one
        print(f"prompt of {y:5d} tokens on {args.devices} stages: k = {k:2d}, sub-sequences {lens}, "
              f"estimated {lat:.3f} ms (unsplit: {one:.3f} ms)")


if __name__ == "__main__":
    main()
