"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the host code, run on the CPU: the C oracle (every entry
point, on buffers of exactly the documented sizes) and the library's host-only logic (argument validation, cache
bookkeeping, the planner's dynamic programs).  GPU code is not instrumented; no kernel is launched."""
import os
import shutil
import struct
import subprocess

import numpy as np
import pytest

import oracle
from paper_2504_08242_amd import build as jbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "sanitize")
OUT = os.path.join(ROOT, "_build", "sanitize")
SAN_ENV = dict(os.environ, ASAN_OPTIONS="abort_on_error=0:detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1")
NAMES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "g_attn", "g_mlp")


def run(cmd, **kw):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert p.returncode == 0, " ".join(cmd) + "\n" + p.stdout[-4000:]
    return p.stdout


def test_oracle_under_asan_and_ubsan_matches_the_ordinary_build():
    os.makedirs(OUT, exist_ok=True)
    exe = os.path.join(OUT, "oracle_driver")
    run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
         "-fno-omit-frame-pointer", "-Wall", "-Wextra", os.path.join(ROOT, "oracle", "jupiter_oracle.c"),
         os.path.join(HERE, "oracle_driver.c"), "-o", exe, "-lm"])
    cfg = dict(n_layers=2, d_model=32, n_heads=2, head_dim=16, d_ffn=40, rms_eps=1e-5, rope_theta=1e4)
    chunks, parents = [3, 1, 5], [-1, 0, 0, 1, 3, -1]
    n_total, n_tree = sum(chunks), len(parents)
    cap = n_total + n_tree                                  # the cache is exactly full after the tree
    rng = np.random.default_rng(7)
    d, f = cfg["d_model"], cfg["d_ffn"]
    shapes = dict(wq=(d, d), wk=(d, d), wv=(d, d), wo=(d, d), w_gate=(f, d), w_up=(f, d), w_down=(d, f),
                  g_attn=(d,), g_mlp=(d,))
    layers = [{n: (rng.standard_normal(shapes[n]) * (0.2 if len(shapes[n]) == 2 else 1.0)).astype(np.float32)
               for n in NAMES} for _ in range(cfg["n_layers"])]
    hidden = rng.standard_normal((n_total + n_tree, d)).astype(np.float32)
    header = [cfg["n_layers"], d, cfg["n_heads"], cfg["head_dim"], f, n_total, cap, len(chunks)]
    header += chunks + [0] * (8 - len(chunks)) + [n_tree] + parents + [0] * (16 - n_tree)
    inp, outp = os.path.join(OUT, "oracle_in.bin"), os.path.join(OUT, "oracle_out.bin")
    with open(inp, "wb") as fh:
        fh.write(struct.pack("<33i", *header))
        for w in layers:
            for n in NAMES:
                fh.write(w[n].tobytes())
        fh.write(hidden.tobytes())
    text = run([exe, inp, outp], env=SAN_ENV)
    assert "oracle_driver ok" in text, text
    got = np.fromfile(outp, dtype=np.float32)
    # the ordinary (-O3, FMA) build on the same numbers: same values up to fp64 rounding order
    ora = oracle.OracleStage(cfg, layers, cap)
    want, pos = [], 0
    for n in chunks:
        want.append(ora.prefill_chunk(hidden[pos:pos + n], pos))
        pos += n
    want.append(ora.prefill_tree(hidden[pos:], parents, pos))
    want = np.concatenate(want)
    n_out = want.size
    assert np.allclose(got[:n_out].reshape(want.shape), want, rtol=1e-5, atol=1e-6)
    assert np.allclose(got[n_out:n_out + ora.kv.size].reshape(ora.kv.shape), ora.kv, rtol=1e-5, atol=1e-6)


def test_library_host_logic_under_asan_and_ubsan():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc is not installed")
    os.makedirs(OUT, exist_ok=True)
    plain = [os.path.join(jbuild.CSRC, s.replace(".hip", ".o")) for s in jbuild.SOURCES]
    if not all(os.path.exists(o) for o in plain):
        jbuild.build_library()
    san_flags = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                 "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer"]
    base = [f for f in jbuild.HIPCC_FLAGS if f not in ("-O3", "-fvisibility=hidden")] + ["-O1", "-g"]
    objs = []
    for src in ("jup_api.hip", "jup_plan.hip"):               # the two sources that are host code only
        obj = os.path.join(OUT, src.replace(".hip", ".o"))
        run([hipcc, *base, *san_flags, "-c", os.path.join(jbuild.CSRC, src), "-o", obj])
        objs.append(obj)
    drv = os.path.join(OUT, "host_driver.o")
    run([hipcc, "-O1", "-g", "-std=c++20", "-I", os.path.join(ROOT, "include"), "-fsanitize=address,undefined",
         "-fno-sanitize-recover=all", "-fno-gpu-sanitize", "-c", os.path.join(HERE, "host_driver.cpp"), "-o", drv])
    rest = [o for o in plain if os.path.basename(o) not in ("jup_api.o", "jup_plan.o")]
    exe = os.path.join(OUT, "host_driver")
    run([hipcc, "--offload-arch=gfx950", "-fsanitize=address,undefined", "-fno-gpu-sanitize", drv, *objs, *rest, "-o", exe])
    text = run([exe], env=SAN_ENV)
    assert "host_driver ok" in text, text
