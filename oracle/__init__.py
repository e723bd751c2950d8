"""ctypes front end of ``jupiter_oracle.c`` -- TEST INFRASTRUCTURE.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package; it imports nothing from the HIP path.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "jupiter_oracle.c")
_LIB = os.path.join(_HERE, "libjupiter_oracle.so")

WEIGHT_NAMES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "g_attn", "g_mlp")

_lib = None


def build(force=True):
    """Compile the oracle with gcc.

    ``x86-64-v3`` (AVX2 + FMA) rather than ``native``: the library is built on
    one machine and may be loaded on another.
    """
    if not force and os.path.exists(_LIB):
        return _LIB
    cmd = ["gcc", "-O3", "-march=x86-64-v3", "-fopenmp", "-std=c11", "-shared", "-fPIC", "-Wall", "-Wextra",
           _SRC, "-o", _LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        L = ctypes.CDLL(_LIB)
        fp = ctypes.POINTER(ctypes.c_float)
        L.oracle_stage_prefill_chunk.restype = ctypes.c_int
        L.oracle_stage_prefill_chunk.argtypes = [
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_double,
            ctypes.POINTER(fp), fp, ctypes.c_int, ctypes.c_int, fp, ctypes.c_int, fp]
        L.oracle_stage_prefill_tree.restype = ctypes.c_int
        L.oracle_stage_prefill_tree.argtypes = [
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_double,
            ctypes.POINTER(fp), fp, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_int32), fp, ctypes.c_int, fp]
        L.oracle_num_threads.restype = ctypes.c_int
        L.oracle_rmsnorm.restype = None
        L.oracle_rmsnorm.argtypes = [fp, fp, fp, ctypes.c_int, ctypes.c_int, ctypes.c_double]
        L.oracle_rope.restype = None
        L.oracle_rope.argtypes = [fp, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_int64), ctypes.c_double]
        L.oracle_linear_nt.restype = None
        L.oracle_linear_nt.argtypes = [fp, fp, fp, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        _lib = L
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def num_threads():
    return int(lib().oracle_num_threads())


class OracleStage:
    """Host-side stage: fp32 weights plus an fp32 KV cache in the contract layout.

    cfg: dict with n_layers, d_model, n_heads, head_dim, d_ffn, rms_eps, rope_theta.
    layers: list (one per layer) of dicts keyed by WEIGHT_NAMES.
    """

    def __init__(self, cfg, layers, max_positions):
        self.cfg = dict(cfg)
        assert len(layers) == cfg["n_layers"]
        self._keep = []
        ptrs = (ctypes.POINTER(ctypes.c_float) * (9 * max(1, len(layers))))()
        for li, w in enumerate(layers):
            for wi, name in enumerate(WEIGHT_NAMES):
                arr, p = _f32(w[name])
                self._keep.append(arr)
                ptrs[li * 9 + wi] = p
        self._ptrs = ptrs
        self.max_positions = int(max_positions)
        self.kv = np.zeros((cfg["n_layers"], 2, cfg["n_heads"], self.max_positions, cfg["head_dim"]), dtype=np.float32)
        self.kv_len = 0

    def reset(self):
        self.kv_len = 0

    def prefill_chunk(self, hidden_in, pos_offset=None, parents=None):
        """One sub-sequence; with ``parents`` (one index per token, -1 or an earlier token) a token tree."""
        c = self.cfg
        hin, hin_p = _f32(hidden_in)
        n = hin.shape[0]
        assert hin.shape == (n, c["d_model"])
        if pos_offset is None:
            pos_offset = self.kv_len
        out = np.empty_like(hin)
        head = (c["n_layers"], c["d_model"], c["n_heads"], c["head_dim"], c["d_ffn"], float(c["rms_eps"]),
                float(c["rope_theta"]), self._ptrs, hin_p, n, int(pos_offset))
        tail = (self.kv.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), self.max_positions,
                out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
        if parents is None:
            rc = lib().oracle_stage_prefill_chunk(*head, *tail)
        else:
            par = np.ascontiguousarray(parents, dtype=np.int32)
            assert par.shape == (n,)
            rc = lib().oracle_stage_prefill_tree(*head, par.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), *tail)
        if rc != 0:
            raise RuntimeError(f"oracle stage forward failed with {rc}")
        self.kv_len = int(pos_offset) + n
        return out

    def prefill_tree(self, hidden_in, parents, pos_offset=None):
        return self.prefill_chunk(hidden_in, pos_offset, parents=parents)

    def keep(self, base_len, slots):
        """Sec. V-A, removal of the rejected candidates: the cache keeps positions below ``base_len`` and,
        behind them, the entries at ``base_len + slots[j]`` (in this order); everything else is dropped."""
        slots = [int(s) for s in slots]
        assert all(0 <= s and base_len + s < self.kv_len for s in slots)
        kept = self.kv[:, :, :, [base_len + s for s in slots], :].copy()
        self.kv[:, :, :, base_len:base_len + len(slots), :] = kept
        self.kv_len = base_len + len(slots)


def rmsnorm(x, g, eps):
    x, xp = _f32(x)
    g, gp = _f32(g)
    y = np.empty_like(x)
    lib().oracle_rmsnorm(xp, gp, y.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), x.shape[0], x.shape[1], float(eps))
    return y


def rope(v, positions, theta):
    """v: [n_vec, dh] rotated in a copy; positions: [n_vec] absolute positions."""
    v = np.array(v, dtype=np.float32, order="C", copy=True)
    pos = np.ascontiguousarray(positions, dtype=np.int64)
    lib().oracle_rope(v.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), v.shape[0], v.shape[1],
                      pos.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), float(theta))
    return v


def linear_nt(x, w):
    x, xp = _f32(x)
    w, wp = _f32(w)
    y = np.empty((x.shape[0], w.shape[0]), dtype=np.float32)
    lib().oracle_linear_nt(xp, wp, y.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), x.shape[0], w.shape[0],
                           x.shape[1])
    return y
