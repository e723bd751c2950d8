#!/usr/bin/env python3
"""Benchmark of the stage kernel: prefill tokens/s of one pipeline stage on one MI355X.

Default workload (the one the headline metric is quoted on): the 8-layer Llama-2-7B-shaped bf16 stage
processes a 2048-token prompt chunk by chunk (4 chunks of 512), every chunk attending to the cached prefix
of the earlier ones.  A step is one pass of the whole hot path over that prompt.  Inputs are seeded synthetic
tensors (hidden ~ N(0,1), weights ~ N(0, 0.02^2)) already resident in HBM when the timed region starts.

A step feeds the prompt with one jup_stage_prefill_chunk call per chunk, one after the other on one stream: the
situation of every pipeline stage but the first, which receives a sub-sequence when its neighbour has finished it
(Sec. IV-A.2), and the definition of the paper's latency function q(x, y) (Sec. IV-B.2).  `value` is the tokens/s of
those steps.  Beside it the JSON line carries
  per_call    every call bracketed by an event pair: median milliseconds per chunk index (q(chunk, c * chunk)) and
              tokens/s = sum of tokens / sum of call times;
  overlapped  the same prompt fed with ONE jup_stage_prefill_chunks call whose consecutive chunks overlap on up to four
              streams (possible where all chunks are at hand, i.e. at a pipeline's first stage); --no-overlap skips it;
  clock_mhz   the shader clock the chip held during the timed steps (a one-wave probe kernel on a second stream);
  roofline    the dominant kernel (the gate/up GEMM with the SwiGLU epilogue), timed in place with HIP events;
  cpu_baseline  the CPU oracle timed on this machine's host cores on a bounded sample of the same workload.
--calibrate-mfma adds `mfma_calibration`: what a bare MFMA loop on random operands sustains on this chip.
--calibrate-fill adds `fill_calibration`: what the operand-fill path of the projection kernels (direct global->LDS
loads of L2-resident data) moves, by bytes in flight, what the same loads stream out of HBM when every byte is read
once (the floor of a short-chunk projection: by grid size, and per launch by bytes moved), and the LDS read rate of a CU.

Prints ONE JSON line.

--workload selects the other benchmark configurations (same JSON line; they are reporting runs, the
default is the metric):
  c3  (default) 7B-shaped stage, 2048-token prompt, --chunk 128|256|512|2048
  c2  7B-shaped stage, 512-token prompt in 8 chunks of 64            (bound by streaming the weights)
  c4  13B-shaped 10-layer stage, 1024-token prompt in 8 chunks of 128 (bound by streaming the weights)
  c5  7B-shaped stage, 8 branches sharing a 512-token prefix, 64 private tokens each; a step is one
      5-token chunk at position 576 on every branch                  (decode-sized, bound by the weights)
  long  7B-shaped stage, one decoding step of a long sequence: a 5-token chunk (1 token + 4 drafts) behind
      --prefix cached positions (default 8192)                        (bound by the weights and the cached keys/values)
  tree  7B-shaped stage, one speculative step: a 64-candidate token tree verified at position 576 in one
      call, then the accepted path kept in the cache                  (bound by the weights)
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0      # MI355X HBM3E
# HBM bytes per launch of the dominant kernel come from the rocprofv3 FETCH_SIZE / WRITE_SIZE summary under
# profiles/ (runs of this script, scaled by a 256 MiB copy: --calibrate-copy); its TRAFFIC lines are keyed by
# workload, chunk size and the kernel instantiation the counters were read for.
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "bench_7b_prompt2048_chunk512_hbm_traffic.txt")


def read_traffic(path, workload, chunk, kernel):
    """Bytes per launch from a line `TRAFFIC workload=c3 chunk=512 kernel=<name> fetch_kib=.. fetch_factor=..
    write_kib=.. write_factor=..`, or None when the table has no line for this kernel instantiation (the counters
    were then read for another tiling and say nothing about this one)."""
    try:
        lines = open(path).read().splitlines()
    except OSError:
        return None
    for line in lines:
        if not line.startswith("TRAFFIC "):
            continue
        kv = dict(item.split("=", 1) for item in line.split()[1:])
        if kv.get("workload") == workload and kv.get("chunk") == str(chunk) and kv.get("kernel") == kernel:
            return (float(kv["fetch_kib"]) * float(kv["fetch_factor"]) +
                    float(kv["write_kib"]) * float(kv["write_factor"])) * 1024.0
    return None


def flops_per_call(cfg, n, p):
    """Algorithmic FLOPs of one chunk call: GEMMs plus causal pairs only."""
    d, f, L = cfg["d_model"], cfg["d_ffn"], cfg["n_layers"]
    gemm = 2.0 * n * (4 * d * d + 3 * d * f)
    attn = 4.0 * d * (n * p + n * (n + 1) / 2)
    return L * (gemm + attn)


W4_BYTES_PER_WEIGHT = 0.5 + 4.0 / 128  # a 4-bit code plus one fp32 scale per 128 weights


def bytes_per_call(cfg, n, p, bytes_per_weight=2.0):
    """Algorithmic HBM bytes of one chunk call: weights once, cached prefix read, new K/V written, hidden in/out."""
    d, f, L = cfg["d_model"], cfg["d_ffn"], cfg["n_layers"]
    weights = bytes_per_weight * L * (4 * d * d + 3 * d * f)
    kv_read = L * 2.0 * (p + n) * d * 2
    kv_write = L * 2.0 * n * d * 2
    return weights + kv_read + kv_write + 2.0 * n * d * 2


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", choices=("c2", "c3", "c4", "c5", "tree", "long"), default="c3")
    ap.add_argument("--prefix", type=int, default=8192, help="workload long: cached positions before the 5-token chunk")
    ap.add_argument("--chunk", type=int, default=512, help="chunk size of workload c3 (128, 256, 512 or 2048)")
    ap.add_argument("--batched", action="store_true",
                    help="workload c5: all 8 branches in one jup_stage_prefill_branches call per step")
    ap.add_argument("--w4", action="store_true",
                    help="the stage holds its projection matrices as 4-bit codes with group-wise scales (dtype "
                         "JUP_BF16_W4), the precision the paper runs its models in.  Calls of up to 64 rows (workloads "
                         "c5, tree, long) stream the codes; a stage made for longer chunks also keeps a bf16 copy of "
                         "the matrices (jup_stage_config_t.w4_expanded) and runs the bf16 kernels on it")
    ap.add_argument("--w4-codes-only", action="store_true",
                    help="with --w4: no bf16 copy, chunks of more than 64 rows take one pass over the codes per 64 rows")
    ap.add_argument("--no-overlap", action="store_true",
                    help="skip the `overlapped` leg (one jup_stage_prefill_chunks call whose consecutive chunks overlap "
                         "on several streams); profiling runs use this, so that every kernel's duration is its own")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="also time torch.matmul (the vendor GEMM library, no fused epilogue) on the four projection "
                         "shapes of the workload's chunk and report it as `vendor_gemm`: context for the per-kernel times")
    ap.add_argument("--calibrate-mfma", action="store_true",
                    help="also run a bare MFMA loop on random operands for about 150 ms and report what it sustains "
                         "(TFLOP/s, the shader clock it held) as `mfma_calibration`")
    ap.add_argument("--calibrate-fill", action="store_true",
                    help="also run the operand-fill probe (direct global->LDS loads from L2, 1 to 16 pieces of 1 KB per "
                         "wave in flight), the HBM stream probe (disjoint regions read once) and the LDS read probe, and report "
                         "them as `fill_calibration`")
    ap.add_argument("--lanes", type=int, default=4,
                    help="lanes enabled for the overlapped call (2..4; for chunks above 256 tokens the library uses all "
                         "of them only when the number of chunks is a multiple of four, else two)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=1024,
                    help="the oracle is timed on the first this-many tokens of the prompt, fed in the same chunks")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 256 MiB device-to-device copy (a kernel of known traffic, for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build covers one GPU (one stage of the pipeline); run with --gpus 1")

    import numpy as np
    import torch

    from paper_2504_08242_amd import binding as jb
    from paper_2504_08242_amd import synth_inputs as si

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    wl = args.workload
    if wl == "c3":
        cfg, prompt, chunk, seed = si.LLAMA7B_STAGE, 2048, args.chunk, 30
        if prompt % chunk:
            sys.exit("bench.py: --chunk must divide 2048")
        what = (f"configs[2]: 8-layer stage of Llama-2-7B shape (d 4096, 32 heads x 128, FFN 11008), "
                f"{prompt}-token prompt as {prompt // chunk} chunks of {chunk}")
    elif wl == "c2":
        cfg, prompt, chunk, seed = si.LLAMA7B_STAGE, 512, 64, 20
        what = "configs[1]: 8-layer stage of Llama-2-7B shape, 512-token prompt as 8 chunks of 64"
    elif wl == "c4":
        cfg, prompt, chunk, seed = si.LLAMA13B_STAGE, 1024, 128, 40
        what = ("configs[3]: 10-layer stage of Llama-2-13B shape (d 5120, 40 heads x 128, FFN 13824), "
                "1024-token prompt as 8 chunks of 128")
    elif wl == "long":
        if args.prefix < 512 or args.prefix % 512:
            sys.exit("bench.py: --prefix must be a positive multiple of 512")
        cfg, prompt, chunk, seed = si.LLAMA7B_STAGE, args.prefix, 512, 80
        what = (f"decoding step of a long sequence on the 8-layer stage of Llama-2-7B shape: one 5-token chunk (1 token + 4 "
                f"drafts) behind {prompt} cached positions")
    elif wl == "tree":
        cfg, prompt, chunk, seed = si.LLAMA7B_STAGE, 576, 64, 70
        what = ("speculative step on the 8-layer stage of Llama-2-7B shape: a 64-candidate token tree verified in one "
                "call at position 576, then the accepted path kept in the cache")
    else:
        cfg, prompt, chunk, seed = si.LLAMA7B_STAGE, 512, 128, 50
        what = ("configs[4]: 8-layer stage of Llama-2-7B shape, 8 branches sharing a 512-token prefix with 64 "
                "private tokens each; a step = one 5-token chunk at position 576 on every branch")
    n_chunks = prompt // chunk
    sdt = "w4" if args.w4 else "bf16"
    # rows of the longest call of the workload decide which copy of the weights a 4-bit stage reads
    w4_expanded = args.w4 and not args.w4_codes_only and wl in ("c2", "c3", "c4") and chunk > 64
    wbytes = W4_BYTES_PER_WEIGHT if args.w4 and not w4_expanded else 2.0

    t0 = time.time()
    hidden_np = si.make_hidden(cfg, seed, prompt, bf16=True)
    if args.w4:
        what += "; projection matrices as 4-bit codes with one fp32 scale per 128 weights"
        if w4_expanded:
            what += (", plus their bf16 expansion (2 more bytes per weight resident), which the bf16 kernels read for "
                     "these chunks of more than 64 rows")
        layers_w4 = si.make_w4_layers(cfg, seed, n_threads=16)
        stage = jb.Stage(cfg, "w4", jb.upload_w4_layers(layers_w4), chunk, w4_expanded=w4_expanded)
    else:
        layers_np = si.make_layers(cfg, seed, bf16=True, n_threads=16)
        stage = jb.Stage(cfg, "bf16", jb.upload_layers(layers_np, "bf16"), chunk)
    kv = jb.KvCache(cfg, sdt, prompt + (chunk if wl in ("tree", "long") else 0))
    hidden = torch.from_numpy(hidden_np).to("cuda:0", torch.bfloat16)
    out = torch.empty_like(hidden)

    if wl == "c5":
        # Untimed set-up: the shared prefix, then 64 private tokens per branch.
        n_branches, n_private, n_step, p_step = 8, 64, 5, 576
        for c in range(n_chunks):
            stage.prefill_chunk(hidden[c * chunk:(c + 1) * chunk], c * chunk, kv)
        branches = [kv.fork(prompt, prompt + n_private + n_step) for _ in range(n_branches)]

        def dev(n, tag):
            return torch.from_numpy(si.make_hidden(cfg, seed, n, tag=tag, bf16=True)).to("cuda:0", torch.bfloat16)

        priv = [dev(n_private, 100 + b) for b in range(n_branches)]
        step_in = [dev(n_step, 200 + b) for b in range(n_branches)]
        step_out = [torch.empty_like(x) for x in step_in]
        for b in range(n_branches):
            stage.prefill_chunk(priv[b], prompt, branches[b])
        calls = [(n_step, p_step)] * n_branches
        tokens_per_step = n_branches * n_step
        if args.batched:
            what += "; all branches in one batched call (the weights are streamed once per step, not once per branch)"
            all_in = torch.cat(step_in)
            all_out = torch.empty_like(all_in)

            def step():  # pos_offset below the length = drop what the last step appended
                stage.prefill_branches(all_in, n_step, [p_step] * n_branches, branches, hidden_out=all_out)
        else:
            def step():
                for b in range(n_branches):
                    stage.prefill_chunk(step_in[b], p_step, branches[b], hidden_out=step_out[b])
    elif wl == "long":
        for c in range(n_chunks):  # untimed: the sequence so far
            stage.prefill_chunk(hidden[c * chunk:(c + 1) * chunk], c * chunk, kv)
        step_in = torch.from_numpy(si.make_hidden(cfg, seed, 5, tag=1, bf16=True)).to("cuda:0", torch.bfloat16)
        step_out = torch.empty_like(step_in)
        calls = [(5, prompt)]
        tokens_per_step = 5

        def step():  # pos_offset below the length = drop what the last step appended
            stage.prefill_chunk(step_in, prompt, kv, hidden_out=step_out)
    elif wl == "tree":
        for c in range(n_chunks):  # untimed: the sequence so far
            stage.prefill_chunk(hidden[c * chunk:(c + 1) * chunk], c * chunk, kv)
        parents = si.make_token_tree(chunk, seed)
        paths = []
        for t, par in enumerate(parents):
            paths.append((paths[par] if par >= 0 else []) + [t])
        accepted = max(paths, key=len)
        cand = torch.from_numpy(si.make_hidden(cfg, seed, chunk, tag=1, bf16=True)).to("cuda:0", torch.bfloat16)
        cand_out = torch.empty_like(cand)
        calls = [(chunk, prompt)]
        tokens_per_step = chunk
        tree_pairs = chunk * prompt + sum(len(pth) for pth in paths)  # prefix plus ancestors and self

        def step():  # the next step's tree overwrites what this one kept
            stage.prefill_tree(cand, prompt, parents, kv, hidden_out=cand_out)
            kv.keep(prompt, accepted)
    else:
        calls = [(chunk, c * chunk) for c in range(n_chunks)]
        tokens_per_step = prompt

        def step_sequential():
            kv.reset()
            for c in range(n_chunks):
                lo = c * chunk
                stage.prefill_chunk(hidden[lo:lo + chunk], lo, kv, hidden_out=out[lo:lo + chunk])

        step = step_sequential
        step_overlapped = None
        if not args.no_overlap and n_chunks >= 2 and not (args.w4 and not w4_expanded):
            stage.enable_overlap(args.lanes)
            # the library's lane rule (jup_stage_prefill_chunks)
            lanes_used = min(2 if chunk > 256 and n_chunks % 4 else args.lanes, n_chunks)

            def step_overlapped():
                kv.reset()
                stage.prefill_chunks(hidden, [chunk] * n_chunks, 0, kv, hidden_out=out)
        what += "; one jup_stage_prefill_chunk call per chunk, one after the other"
    if wl in ("c5", "tree", "long"):
        step_overlapped = None
    torch.cuda.synchronize()
    print(f"[bench] inputs ready in {time.time() - t0:.1f}s", file=sys.stderr, flush=True)

    if args.calibrate_copy:
        src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def timed(fn, probe=False):
        """args.warmup untimed and args.steps timed runs of fn; (seconds, clock in MHz or None).  With probe, a
        one-wave kernel on a second stream reads the shader clock against the 100 MHz reference clock for about 80 % of
        the timed region."""
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        ticks = None
        if probe:
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            one = time.perf_counter() - t0
            ticks = torch.zeros(2, dtype=torch.int64, device="cuda:0")
            side = torch.cuda.Stream()
            torch.cuda.synchronize()
            jb.diag_clock_probe(max(int(0.8 * one * args.steps * 1e8), 1000), ticks, stream=side)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.current_stream().synchronize()
        dt = time.perf_counter() - t0
        torch.cuda.synchronize()
        mhz = None
        if ticks is not None:
            t = ticks.cpu().tolist()
            mhz = round(100.0 * t[0] / max(t[1], 1), 1)
        return dt, mhz

    mfma_calibration = None
    if args.calibrate_mfma:
        ops = torch.randn(1 << 19, device="cuda:0").to(torch.bfloat16)   # 1 MiB of random bf16 values
        n_wg, ticks, sink = 256, torch.zeros((256, 2), dtype=torch.int64, device="cuda:0"), torch.zeros(1, device="cuda:0")
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        iters = 20000
        for _ in range(2):   # the second launch is sized from the first so that it lasts about 150 ms
            ev[0].record()
            flop = jb.diag_mfma_loop(ops, n_wg, iters, ticks, sink)
            ev[1].record()
            torch.cuda.synchronize()
            ms = ev[0].elapsed_time(ev[1])
            last_iters, iters = iters, max(int(iters * 150.0 / max(ms, 1e-3)), 1000)
        t = ticks.cpu().numpy().astype("float64")
        mfma_calibration = {"kernel": "bare loop of v_mfma_f32_32x32x16_bf16 on random operands, 256 workgroups x 8 waves "
                                      "(two per SIMD), 8 independent accumulators per wave",
                            "ms": round(ms, 2), "iters_per_wave": last_iters, "tflops": round(flop / ms / 1e9, 1),
                            "frac_of_published_peak": round(flop / ms / 1e9 / PEAK_BF16_TFLOPS, 4),
                            "clock_mhz_mean": round(float(100.0 * (t[:, 0] / t[:, 1]).mean()), 1),
                            "clock_mhz_min": round(float(100.0 * (t[:, 0] / t[:, 1]).min()), 1)}
        del ops

    fill_calibration = None
    if args.calibrate_fill:
        window = torch.ones(16 << 20, dtype=torch.uint8, device="cuda:0")   # every workgroup walks these 16 MiB: L2 hits
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        by_depth = {}
        for depth in (1, 2, 4, 8, 16):
            best = None
            for _ in range(4):
                ev[0].record()
                nbytes = jb.diag_fill_probe(window, 256, depth, 4096)
                ev[1].record()
                torch.cuda.synchronize()
                ms = ev[0].elapsed_time(ev[1])
                best = ms if best is None else min(best, ms)
            by_depth[f"{8 * depth}-{16 * depth} KB in flight per CU"] = round(nbytes / best / 1e9, 2)
        lds = {}
        ticks, sink = torch.zeros(256, dtype=torch.int64, device="cuda:0"), torch.zeros(1, dtype=torch.int32, device="cuda:0")
        for threads in (256, 512, 1024):
            for _ in range(2):
                per_wg = jb.diag_lds_read_probe(256, threads, 2000, ticks, sink)
                torch.cuda.synchronize()
            lds[f"{threads // 64} waves"] = round(per_wg / float(ticks.cpu().numpy().astype("float64").mean()), 1)
        # the weight stream of a short-chunk projection with everything else taken away: disjoint regions, read once
        big = torch.ones(2 << 30, dtype=torch.uint8, device="cuda:0")
        seg = 256 << 20   # bytes of the launches timed by grid size; the 2 GiB buffer keeps every launch cold
        def stream_launches(n_launch, n_wg, ppw):   # back to back on the stream, like the kernels of a call
            ev[0].record()
            nb = jb.diag_stream_probe(big, n_wg, 4, ppw, n_launch)
            ev[1].record()
            torch.cuda.synchronize()
            return nb, ev[0].elapsed_time(ev[1]) / n_launch
        by_grid = {}
        for n_wg in (128, 192, 230, 256):
            ppw = (seg // n_wg // 8192) // 4 * 4
            best = min(stream_launches(8, n_wg, ppw)[1] for _ in range(3))
            by_grid[f"{n_wg} workgroups"] = round(n_wg * ppw * 8192 / best / 1e9, 2)
        by_size = {}
        for ppw in (4, 12, 16, 24, 44, 48, 88):   # x 256 workgroups x 8 KiB: 8.4 .. 184.5 MB, the projections' weight bytes
            best = min(stream_launches(32, 256, ppw)[1] for _ in range(3))
            by_size[f"{256 * ppw * 8192 / 1e6:.1f} MB"] = round(1e3 * best, 2)
        del big
        fill_calibration = {"hbm_to_lds_tb_per_s": by_grid, "hbm_to_lds_launch_us_256_workgroups": by_size,
                            "l2_to_lds_tb_per_s": by_depth,
                            "what": "256 workgroups x 8 waves copy 1 KB pieces of a 16 MiB window into LDS with direct "
                                    "global->LDS loads (best of 4 launches of 8 GiB each); LDS read: 16 bytes per lane and "
                                    "instruction, conflict-free, bytes per shader clock and CU; hbm_to_lds: workgroups of "
                                    "8 waves stream disjoint regions once (4 pieces of 1 KB per wave in flight), rate of "
                                    "256 MiB launches by grid size and microseconds per launch by bytes moved, launches "
                                    "enqueued back to back like the kernels of a call",
                            "lds_read_bytes_per_clk_per_cu": lds}
        del window

    vendor_gemm = None
    if args.vendor_gemm:
        d_, f_, m_ = cfg["d_model"], cfg["d_ffn"], calls[0][0]
        vendor_gemm = {"what": "torch.matmul (vendor library) on bf16 random operands, plain product without any epilogue, "
                               "average of 50 back-to-back launches between two events", "rows": m_}
        for name, nn, kk in (("gemm_qkv", 3 * d_, d_), ("gemm_o", d_, d_), ("gemm_gate_up", 2 * f_, d_), ("gemm_down", d_, f_)):
            xa = torch.randn(m_, kk, device="cuda:0").to(torch.bfloat16)
            xw = (torch.randn(nn, kk, device="cuda:0") * 0.02).to(torch.bfloat16)
            for _ in range(5):
                xc = xa @ xw.t()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            torch.cuda.synchronize()
            ev[0].record()
            for _ in range(50):
                xc = xa @ xw.t()
            ev[1].record()
            torch.cuda.synchronize()
            us = ev[0].elapsed_time(ev[1]) / 50 * 1e3
            vendor_gemm[name] = {"us": round(us, 2), "tflops": round(2.0 * m_ * nn * kk / us / 1e6, 1)}
            del xa, xw, xc

    elapsed, clock_mhz = timed(step, probe=True)
    out_timed = out.clone() if wl in ("c2", "c3", "c4") else None  # what the timed steps wrote (the passes below reuse out)
    ms_per_step = elapsed / args.steps * 1e3
    tokens_per_s = tokens_per_step * args.steps / elapsed
    step_flops = sum(flops_per_call(cfg, n, p) for n, p in calls)
    if wl == "tree":  # pairs a query really has: prefix, ancestors, itself (not the causal triangle)
        step_flops += cfg["n_layers"] * 4.0 * cfg["d_model"] * (tree_pairs - (chunk * prompt + chunk * (chunk + 1) / 2))
    step_bytes = sum(bytes_per_call(cfg, n, p, wbytes) for n, p in calls)
    if wl == "c5" and args.batched:  # one pass over the weights serves every branch
        d_, f_, L_ = cfg["d_model"], cfg["d_ffn"], cfg["n_layers"]
        step_bytes -= (len(calls) - 1) * wbytes * L_ * (4 * d_ * d_ + 3 * d_ * f_)
    step_tflops = step_flops / (ms_per_step * 1e-3) / 1e12
    step_gbs = step_bytes / (ms_per_step * 1e-3) / 1e9

    # q(x, y) of Sec. IV-B.2: every call between two events on the stream it runs on, median over the steps.
    per_call = None
    if wl in ("c2", "c3", "c4"):
        evs = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_chunks)]
               for _ in range(args.steps)]
        for rep in range(args.steps):
            kv.reset()
            for c in range(n_chunks):
                lo = c * chunk
                evs[rep][c][0].record()
                stage.prefill_chunk(hidden[lo:lo + chunk], lo, kv, hidden_out=out[lo:lo + chunk])
                evs[rep][c][1].record()
        torch.cuda.synchronize()
        ms_chunk = [float(np.median([evs[rep][c][0].elapsed_time(evs[rep][c][1]) for rep in range(args.steps)]))
                    for c in range(n_chunks)]
        pc_s = sum(ms_chunk) * 1e-3
        per_call = {"what": "one jup_stage_prefill_chunk call between two events, median over the steps; chunk c is "
                            "q(chunk_tokens, c * chunk_tokens)",
                    "ms_per_chunk": [round(m, 4) for m in ms_chunk],
                    "tokens_per_s": round(prompt / pc_s, 1),
                    "tflops": round(step_flops / pc_s / 1e12, 1),
                    "frac_of_bf16_mfma_peak": round(step_flops / pc_s / 1e12 / PEAK_BF16_TFLOPS, 4)}

    # The same prompt in one call, consecutive chunks overlapping on several streams.
    overlapped = None
    if step_overlapped is not None:
        # no clock probe here: the process has four hardware queues, the call's four streams take them all, and a probe
        # on a fifth stream would hold one lane's queue for as long as it runs
        o_elapsed, _ = timed(step_overlapped)
        o_ms = o_elapsed / args.steps * 1e3
        overlapped = {"what": f"one jup_stage_prefill_chunks call for the whole prompt, consecutive chunks overlapping on "
                              f"{lanes_used} streams (all chunks at hand: a pipeline's first stage)",
                      "tokens_per_s": round(tokens_per_step * args.steps / o_elapsed, 1), "ms_per_step": round(o_ms, 4),
                      "tflops": round(step_flops / (o_ms * 1e-3) / 1e12, 1),
                      "frac_of_bf16_mfma_peak": round(step_flops / (o_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}

    # Second pass: the same work with an event pair around every launch of one kernel class at a time, the
    # chunks one after the other (overlapping chunks share the GPU, and a kernel's duration would include its wait
    # for the other chunk's kernels).
    trace_step = step
    per_kernel = {}
    for name in ("gemm_gate_up", "gemm_qkv", "gemm_down", "gemm_o", "attention", "rmsnorm"):
        stage.trace(jb.KERNEL_IDS[name], max_launches=4 * cfg["n_layers"] * len(calls) * max(args.steps, 1))
        reps = args.steps if name == "gemm_gate_up" else min(args.steps, 3)
        for _ in range(reps):
            trace_step()
        torch.cuda.synchronize()
        ms, launches, dropped = stage.trace_read()
        per_kernel[name] = {"avg_us": ms / max(launches, 1) * 1e3, "launches_per_step": launches // max(reps, 1),
                            "dropped": dropped}
    stage.trace(-1)
    dom = per_kernel["gemm_gate_up"]
    n_call = calls[0][0] * (len(calls) if wl == "c5" and args.batched else 1)  # rows of one GEMM launch
    d, f = cfg["d_model"], cfg["d_ffn"]
    dom_flops = 2.0 * n_call * (2 * f) * d  # one launch: [n, d] x [2f, d]^T
    dom_bytes = wbytes * 2 * f * d + 2.0 * (n_call * d + n_call * f)  # weights + activations in + activations out
    codes = args.w4 and not w4_expanded  # the projections are the 4-bit kernels
    dom_name = "gemm_w4<gate_up+swiglu>" if codes else stage.kernel_name(jb.KERNEL_IDS["gemm_gate_up"], n_call)
    traffic = None if codes else read_traffic(TRAFFIC_TABLE, wl, chunk, dom_name)
    dom_s = dom["avg_us"] * 1e-6
    # which roof the dominant kernel sits under: the ridge of the chip is peak flop/s over peak byte/s
    if dom_flops / dom_bytes >= PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
        achieved = dom_flops / dom_s / 1e12
        roofline = {"bound": "mfma", "kernel": dom_name, "achieved": round(achieved, 1),
                    "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4)}
    else:
        achieved = dom_bytes / dom_s / 1e9
        roofline = {"bound": "hbm", "kernel": dom_name, "achieved": round(achieved, 1),
                    "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(achieved / PEAK_HBM_GBS, 4)}
    roofline.update({"timed": "event pairs around each launch in a pass that feeds the chunks one call after the other "
                              "(in the overlapped call two chunks share the GPU and a launch waits for its share)",
                     "avg_launch_us": round(dom["avg_us"], 2), "flop_per_launch": dom_flops,
                     "algorithmic_bytes": dom_bytes, "traffic": traffic,
                     "traffic_unit": "HBM bytes per launch",
                     "traffic_source": (os.path.relpath(TRAFFIC_TABLE, ROOT) + " (rocprofv3 FETCH_SIZE / WRITE_SIZE runs of "
                                        "this script for this kernel instantiation)") if traffic else
                                       "no counter reading on file for this kernel instantiation"})

    cpu_baseline = None
    if not args.no_cpu_baseline and wl not in ("c5", "tree", "long"):
        import oracle
        ns = min(max(args.cpu_sample_tokens, 1), prompt)
        if args.w4:  # the oracle of a 4-bit stage runs on the matrices the codes and scales expand to
            from oracle import w4
            layers_np = w4.dequantize_layers(layers_w4)
        ora = oracle.OracleStage(cfg, layers_np, ns)
        ref = np.empty((ns, cfg["d_model"]), np.float32)
        t0 = time.perf_counter()
        for lo in range(0, ns, chunk):
            hi = min(lo + chunk, ns)
            ref[lo:hi] = ora.prefill_chunk(hidden_np[lo:hi], lo)
        dt = time.perf_counter() - t0
        got = out_timed[:ns].float().cpu().numpy().astype(np.float64)
        cpu_baseline = {"value": round(ns / dt, 2), "unit": "tokens/s", "cores": oracle.num_threads(),
                        "kind": "oracle", "seconds": round(dt, 2),
                        "sample": f"first {ns} of the {prompt} prompt tokens in chunks of {chunk}, all "
                                  f"{cfg['n_layers']} layers",
                        "gpu_vs_oracle_rel_l2": float(np.linalg.norm(got - ref) / np.linalg.norm(ref.astype(np.float64)))}

    print(json.dumps({
        "metric": "prefill_tokens_per_s_per_stage",
        "value": round(tokens_per_s, 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16 activations, 4-bit weights" if args.w4 else "bf16",
        "data": "synthetic",
        "config": {"workload": what, "tokens_per_step": tokens_per_step, "chunk_tokens": n_call},
        "tflops": round(step_tflops, 1),
        "frac_of_bf16_mfma_peak": round(step_tflops / PEAK_BF16_TFLOPS, 4),
        "algorithmic_gb_per_s": round(step_gbs, 1),
        "frac_of_hbm_peak": round(step_gbs / PEAK_HBM_GBS, 4),
        "clock_mhz": clock_mhz,
        "per_call": per_call,
        "overlapped": overlapped,
        "mfma_calibration": mfma_calibration,
        "fill_calibration": fill_calibration,
        "vendor_gemm": vendor_gemm,
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "kernels_avg_us": {k: round(v["avg_us"], 2) for k, v in per_kernel.items()},
    }))


if __name__ == "__main__":
    main()
