#!/usr/bin/env python3
"""Measures q(x, y) of a stage on this GPU: the latency of one chunk of x tokens that attends to y cached ones.

The planner of the Jupiter paper (Sec. IV-B.2) picks the chunk lengths of the intra-sequence pipeline from
exactly this function, obtained by profiling the device (Sec. III, step 1), and needs the smallest chunk
length b that still uses the accelerator well.  This script produces that table for one stage held by one
MI355X: rows x (chunk length), columns y (cached prefix), entries in milliseconds, plus tokens/s per row and
the knee of the x -> tokens/s curve.  Timing does not depend on the values, so the cache is filled with
whatever a long synthetic prompt leaves there.

    python -m paper_2504_08242_amd.profile_qxy [--model 7b|13b] [--layers N] [--reps R] [--csv out.csv]
"""
import argparse
import json
import sys
import time


def knee(table, xs, y0, within=0.8):
    """Smallest chunk length whose tokens/s at y = y0 reaches `within` of the best one in the table: the shortest
    sub-sequence b that still uses the accelerator well (Sec. IV-B.2)."""
    rate = {x: x / table[(x, y0)] for x in xs}
    best = max(rate.values())
    return min(x for x in xs if rate[x] >= within * best)


def format_table(table, xs, ys, title):
    """The q(x, y) table as text: one row per x, one column per y (ms), tokens/s at the smallest y, the knee."""
    lines = [title, "x \\ y   " + "".join(f"{y:>10d}" for y in ys) + f"   tokens/s at y={ys[0]}"]
    for x in xs:
        lines.append(f"{x:<8d}" + "".join(f"{table[(x, y)]:10.3f}" for y in ys) + f"   {x / table[(x, ys[0])] * 1e3:12.0f}")
    lines.append(f"smallest chunk within 20 % of the best throughput at y={ys[0]}: b = {knee(table, xs, ys[0])} tokens")
    return "\n".join(lines)


def write_csv(table, path):
    """x,y,ms rows, the file planner.read_qxy_csv() reads."""
    with open(path, "w") as f:
        f.write("x,y,ms\n")
        for (x, y), ms in sorted(table.items()):
            f.write(f"{x},{y},{ms:.4f}\n")


def measure(cfg, xs, ys, reps=5, w4=False, seed=60, progress=None):
    """q(x, y) in milliseconds for every x in xs and y in ys on cuda:0: wall-clock time around `reps` back-to-back
    jup_stage_prefill_chunk calls (one call per entry, no overlap between chunks).  -> {(x, y): ms}."""
    import torch

    from . import binding as jb
    from . import synth_inputs as si

    assert torch.cuda.is_available(), "profile_qxy needs the MI355X"
    xs, ys = sorted(xs), sorted(ys)
    x_max, y_max = xs[-1], ys[-1]
    if w4:
        stage = jb.Stage(cfg, "w4", jb.upload_w4_layers(si.make_w4_layers(cfg, seed, n_threads=16)), x_max)
    else:
        layers_np = si.make_layers(cfg, seed, bf16=True, n_threads=16)
        stage = jb.Stage(cfg, "bf16", jb.upload_layers(layers_np, "bf16"), x_max)
    kv = jb.KvCache(cfg, "bf16", y_max + x_max)
    hidden = torch.from_numpy(si.make_hidden(cfg, seed, x_max, bf16=True)).to("cuda:0", torch.bfloat16)
    out = torch.empty_like(hidden)

    def ensure_len(y):
        """Appends (untimed) until the cache holds at least y positions; the values do not matter for timing."""
        p0 = len(kv)
        while p0 < y:
            m = min(x_max, y - p0)
            stage.prefill_chunk(hidden[:m], p0, kv, hidden_out=out[:m])
            p0 += m
        torch.cuda.synchronize()

    table = {}
    for x in xs:
        for y in ys:
            ensure_len(y)

            def call():  # pos_offset below the cache length = overwrite from there
                stage.prefill_chunk(hidden[:x], y, kv, hidden_out=out[:x])
            call()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                call()
            torch.cuda.synchronize()
            table[(x, y)] = (time.perf_counter() - t0) / reps * 1e3
        if progress:
            progress(x)
    return table


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--model", choices=("7b", "13b"), default="7b")
    ap.add_argument("--layers", type=int, default=0, help="layers of the stage (default: the benchmark stage)")
    ap.add_argument("--x", type=int, nargs="+", default=[16, 32, 64, 128, 256, 384, 512, 768, 1024, 1536, 2048])
    ap.add_argument("--y", type=int, nargs="+", default=[0, 512, 1024, 2048, 4096, 8192])
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--csv", default="")
    ap.add_argument("--w4", action="store_true",
                    help="profile a stage that holds its projection matrices as 4-bit codes (dtype JUP_BF16_W4)")
    args = ap.parse_args()

    from . import synth_inputs as si

    cfg = dict(si.LLAMA7B_STAGE if args.model == "7b" else si.LLAMA13B_STAGE)
    if args.layers:
        cfg["n_layers"] = args.layers
    xs, ys = sorted(args.x), sorted(args.y)
    table = measure(cfg, xs, ys, reps=args.reps, w4=args.w4,
                    progress=lambda x: print(f"[qxy] x={x} done", file=sys.stderr, flush=True))
    print(format_table(table, xs, ys,
                       f"q(x,y) in ms: {args.model} stage of {cfg['n_layers']} layers, "
                       f"{'bf16 activations and 4-bit weights' if args.w4 else 'bf16'}, one MI355X; {args.reps} repetitions each"))
    if args.csv:
        write_csv(table, args.csv)
    print(json.dumps({"model": args.model, "n_layers": cfg["n_layers"], "knee_tokens": knee(table, xs, ys[0]),
                      "q_ms": {f"{x},{y}": round(ms, 4) for (x, y), ms in sorted(table.items())}}))


if __name__ == "__main__":
    main()
