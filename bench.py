#!/usr/bin/env python3
"""Benchmark of the stage kernel: prefill tokens/s of one pipeline stage on one MI355X.

A step is one pass of the whole hot path over one prompt: the 8-layer Llama-2-7B-shaped bf16 stage
processes a 2048-token prompt chunk by chunk (default 4 chunks of 512), every chunk attending to the
cached prefix of the earlier ones.  Inputs are seeded synthetic tensors (hidden ~ N(0,1), weights
~ N(0, 0.02^2)) already resident in HBM when the timed region starts.

Prints ONE JSON line.  `roofline` is for the dominant kernel (the gate/up GEMM with the SwiGLU epilogue),
timed in place with HIP events in a second pass over the same steps; `cpu_baseline` is the CPU oracle
timed on this machine's host cores on a bounded sample of the same workload.
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
# HBM bytes per launch of the dominant kernel at chunk 512, from rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this
# script scaled by a 256 MiB copy (--calibrate-copy); the summary of those runs lies under profiles/.
GATE_UP_TRAFFIC_BYTES = {512: (106863.5 * 2.0 + 11046.2 * 1.0) * 1024}
PROMPT_TOKENS = 2048


def flops_per_call(cfg, n, p):
    """Algorithmic FLOPs of one chunk call: GEMMs plus causal pairs only."""
    d, f, L = cfg["d_model"], cfg["d_ffn"], cfg["n_layers"]
    gemm = 2.0 * n * (4 * d * d + 3 * d * f)
    attn = 4.0 * d * (n * p + n * (n + 1) / 2)
    return L * (gemm + attn)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--chunk", type=int, default=512, help="chunk size (128, 256, 512 or 2048)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=1024,
                    help="the oracle is timed on the first this-many tokens of the prompt, fed in the same chunks")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 256 MiB device-to-device copy (a kernel of known traffic, for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build covers one GPU (one stage of the pipeline); run with --gpus 1")
    if PROMPT_TOKENS % args.chunk:
        sys.exit("bench.py: --chunk must divide 2048")

    import numpy as np
    import torch

    from paper_2504_08242_amd import binding as jb
    from paper_2504_08242_amd import synth_inputs as si

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    cfg = si.LLAMA7B_STAGE
    chunk = args.chunk
    n_chunks = PROMPT_TOKENS // chunk
    seed = 30

    t0 = time.time()
    layers_np = si.make_layers(cfg, seed, bf16=True, n_threads=16)
    hidden_np = si.make_hidden(cfg, seed, PROMPT_TOKENS, bf16=True)
    stage = jb.Stage(cfg, "bf16", jb.upload_layers(layers_np, "bf16"), chunk)
    kv = jb.KvCache(cfg, "bf16", PROMPT_TOKENS)
    hidden = torch.from_numpy(hidden_np).to("cuda:0", torch.bfloat16)
    out = torch.empty_like(hidden)
    torch.cuda.synchronize()
    print(f"[bench] inputs ready in {time.time() - t0:.1f}s", file=sys.stderr, flush=True)

    def step():
        kv.reset()
        for c in range(n_chunks):
            lo = c * chunk
            stage.prefill_chunk(hidden[lo:lo + chunk], lo, kv, hidden_out=out[lo:lo + chunk])

    if args.calibrate_copy:
        src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    tokens_per_s = PROMPT_TOKENS * args.steps / elapsed
    step_flops = sum(flops_per_call(cfg, chunk, c * chunk) for c in range(n_chunks))
    step_tflops = step_flops / (ms_per_step * 1e-3) / 1e12

    # Second pass: the same steps with an event pair around every launch of the dominant kernel.
    per_kernel = {}
    for name in ("gemm_gate_up", "gemm_qkv", "gemm_down", "gemm_o", "attention", "rmsnorm"):
        stage.trace(jb.KERNEL_IDS[name], max_launches=4 * cfg["n_layers"] * n_chunks * max(args.steps, 1))
        reps = args.steps if name == "gemm_gate_up" else min(args.steps, 3)
        for _ in range(reps):
            step()
        torch.cuda.synchronize()
        ms, launches, dropped = stage.trace_read()
        per_kernel[name] = {"avg_us": ms / max(launches, 1) * 1e3, "launches_per_step": launches // max(reps, 1),
                            "dropped": dropped}
    stage.trace(-1)
    dom = per_kernel["gemm_gate_up"]
    dom_flops = 2.0 * chunk * (2 * cfg["d_ffn"]) * cfg["d_model"]  # one launch: [chunk, d] x [2f, d]^T
    achieved = dom_flops / (dom["avg_us"] * 1e-6) / 1e12
    roofline = {"bound": "mfma", "kernel": "gemm_bf16_nt<gate_up+swiglu>", "achieved": round(achieved, 1),
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                "avg_launch_us": round(dom["avg_us"], 2), "flop_per_launch": dom_flops, "traffic": GATE_UP_TRAFFIC_BYTES.get(chunk),
                "traffic_unit": "bytes per launch (offline rocprofv3 counters)",
                "algorithmic_bytes": 2.0 * (2 * cfg["d_ffn"] * cfg["d_model"] + chunk * cfg["d_model"]
                                            + chunk * cfg["d_ffn"])}

    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        ns = min(max(args.cpu_sample_tokens, 1), PROMPT_TOKENS)
        ora = oracle.OracleStage(cfg, layers_np, ns)
        ref = np.empty((ns, cfg["d_model"]), np.float32)
        t0 = time.perf_counter()
        for lo in range(0, ns, chunk):
            hi = min(lo + chunk, ns)
            ref[lo:hi] = ora.prefill_chunk(hidden_np[lo:hi], lo)
        dt = time.perf_counter() - t0
        got = out[:ns].float().cpu().numpy().astype(np.float64)
        cpu_baseline = {"value": round(ns / dt, 2), "unit": "tokens/s", "cores": oracle.num_threads(),
                        "kind": "oracle", "seconds": round(dt, 2),
                        "sample": f"first {ns} of the {PROMPT_TOKENS} prompt tokens in chunks of {chunk}, all "
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
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"configs[2]: 8-layer stage of Llama-2-7B shape (d 4096, 32 heads x 128, FFN 11008), "
                               f"{PROMPT_TOKENS}-token prompt as {n_chunks} chunks of {chunk}",
                   "prompt_tokens": PROMPT_TOKENS, "chunk_tokens": chunk},
        "tflops": round(step_tflops, 1),
        "frac_of_bf16_mfma_peak": round(step_tflops / PEAK_BF16_TFLOPS, 4),
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "kernels_avg_us": {k: round(v["avg_us"], 2) for k, v in per_kernel.items()},
    }))


if __name__ == "__main__":
    main()
