"""Seeded synthetic inputs shared by the tests and the benchmark.

This module holds none of the method's arithmetic: it only draws random
tensors of the shapes of the paper's workloads (Llama-2-7B / 13B decoder
layers, Sec. V-A of the Jupiter paper) and rounds them to bf16 where a run
asks for bf16 storage.  The same arrays are handed to the CPU oracle and to the
HIP library, so neither side generates data for the other.

Recipe
------
* hidden states  ~ N(0, 1)
* weight matrices ~ N(0, 0.02**2)   (0.02 is the standard deviation)
* RMSNorm gains  = 1 + N(0, 0.02**2)  (gains of mean 0 would scale every
  activation by ~0.02; gains of exactly 1 would leave the multiply untested)
* every tensor has a generator of its own,
  ``numpy.random.default_rng([seed, stream, index])`` with
  stream = layer number for weights (index = position in WEIGHT_NAMES) and
  stream = HIDDEN_STREAM for hidden states (index = caller-chosen tag),
  drawn with ``standard_normal(dtype=float32)``; tensors are therefore
  independent of the order in which they are requested.
* token trees (the candidates of a speculative step, Sec. V-A; the paper
  evaluates with Medusa's tree, which has one root, at most 64 nodes and a
  few levels, bushy near the root): ``make_token_tree`` draws, for every
  node after the root, a parent among the earlier nodes of depth below
  ``max_depth`` with probability proportional to 2**(-depth), from
  ``default_rng([seed, TREE_STREAM, n_tokens])``.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np

WEIGHT_NAMES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "g_attn", "g_mlp")
HIDDEN_STREAM = 1_000_000
TREE_STREAM = 2_000_000
W4_STREAM = 3_000_000

# Architectures of the five benchmark configurations.
TINY = dict(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ffn=688, rms_eps=1e-5, rope_theta=1e4)
LLAMA7B_STAGE = dict(n_layers=8, d_model=4096, n_heads=32, head_dim=128, d_ffn=11008, rms_eps=1e-5, rope_theta=1e4)
LLAMA13B_STAGE = dict(n_layers=10, d_model=5120, n_heads=40, head_dim=128, d_ffn=13824, rms_eps=1e-5, rope_theta=1e4)


def weight_shape(cfg, name):
    d, f = cfg["d_model"], cfg["d_ffn"]
    return {"wq": (d, d), "wk": (d, d), "wv": (d, d), "wo": (d, d), "w_gate": (f, d), "w_up": (f, d),
            "w_down": (d, f), "g_attn": (d,), "g_mlp": (d,)}[name]


def round_to_bf16(a):
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    out = ((u + r) & np.uint32(0xFFFF0000)).view(np.float32)
    return out


def bf16_bits(a):
    """Upper 16 bits of fp32 values that are already bf16-representable."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def make_weight(cfg, seed, layer, name, bf16=False, weight_std=0.02):
    idx = WEIGHT_NAMES.index(name)
    rng = np.random.default_rng([seed, layer, idx])
    w = rng.standard_normal(weight_shape(cfg, name), dtype=np.float32)
    if name.startswith("g_"):
        w = np.float32(1.0) + np.float32(0.02) * w
    else:
        w *= np.float32(weight_std)
    return round_to_bf16(w) if bf16 else w


def make_layers(cfg, seed, bf16=False, weight_std=0.02, n_threads=8):
    """List (one entry per layer) of dicts keyed by WEIGHT_NAMES, fp32 arrays."""
    jobs = [(l, n) for l in range(cfg["n_layers"]) for n in WEIGHT_NAMES]
    with ThreadPoolExecutor(max_workers=n_threads) as ex:
        arrs = list(ex.map(lambda j: make_weight(cfg, seed, j[0], j[1], bf16, weight_std), jobs))
    layers = [dict() for _ in range(cfg["n_layers"])]
    for (l, n), a in zip(jobs, arrs):
        layers[l][n] = a
    return layers


def make_hidden(cfg, seed, n_tokens, tag=0, bf16=False):
    rng = np.random.default_rng([seed, HIDDEN_STREAM, tag])
    h = rng.standard_normal((n_tokens, cfg["d_model"]), dtype=np.float32)
    return round_to_bf16(h) if bf16 else h


def make_token_tree(n_tokens, seed, max_depth=4):
    """parents[t] for a one-root tree of n_tokens nodes: -1 for the root, else the index of an earlier node."""
    rng = np.random.default_rng([seed, TREE_STREAM, n_tokens])
    parents = np.full(n_tokens, -1, dtype=np.int32)
    depth = np.zeros(n_tokens, dtype=np.int64)
    for t in range(1, n_tokens):
        ok = np.flatnonzero(depth[:t] < max_depth)
        w = 0.5 ** depth[ok]
        parents[t] = ok[rng.choice(len(ok), p=w / w.sum())]
        depth[t] = depth[parents[t]] + 1
    return parents


def make_w4_layers(cfg, seed, weight_std=0.02, n_threads=8):
    """Seeded 4-bit projection matrices: per layer a dict with, for each of the seven matrices, ``name`` = uint8
    [out, in/2] (two 4-bit codes per byte) and ``name + '_scale'`` = fp32 [out, in/128], plus the two gains
    (fp32, bf16-representable).  Codes are round(2.3 z) + 8 clipped to 0..15 with z ~ N(0,1) and scales are
    weight_std / 2.3 times (0.75 + U(0, 0.5)) rounded to bf16, so that the expanded matrices look like N(0,
    weight_std^2) weights after round-to-nearest 4-bit quantisation.  Bytes and scales come straight from the
    generator: there is no quantiser, hence none to share between the two sides."""
    matrices = [n for n in WEIGHT_NAMES if not n.startswith("g_")]

    def one(job):
        l, name = job
        idx = WEIGHT_NAMES.index(name)
        if name.startswith("g_"):
            return make_weight(cfg, seed, l, name, bf16=True)
        n_out, n_in = weight_shape(cfg, name)
        rng = np.random.default_rng([seed, W4_STREAM, l, idx])
        z = rng.standard_normal((n_out, n_in), dtype=np.float32)
        z *= np.float32(2.3)
        np.rint(z, out=z)
        z += np.float32(8.0)
        np.clip(z, 0.0, 15.0, out=z)
        codes = z.astype(np.uint8)
        packed = codes[:, 0::2] | (codes[:, 1::2] << np.uint8(4))
        u = rng.random((n_out, n_in // 128), dtype=np.float32)
        scale = round_to_bf16(np.float32(weight_std / 2.3) * (np.float32(0.75) + np.float32(0.5) * u))
        return np.ascontiguousarray(packed), scale

    jobs = [(l, n) for l in range(cfg["n_layers"]) for n in WEIGHT_NAMES]
    with ThreadPoolExecutor(max_workers=n_threads) as ex:
        res = list(ex.map(one, jobs))
    layers = [dict() for _ in range(cfg["n_layers"])]
    for (l, n), r in zip(jobs, res):
        if n.startswith("g_"):
            layers[l][n] = r
        else:
            layers[l][n], layers[l][n + "_scale"] = r
    return layers
