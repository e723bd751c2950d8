"""Shared plumbing of the GPU parity tests: the same seeded numpy inputs go to the CPU oracle and to
the HIP library; results come back as numpy fp32."""
import numpy as np

import oracle
from paper_2504_08242_amd import binding as jb
from paper_2504_08242_amd import synth_inputs as si

# Tolerances of the parity bar.
F32_MAX_ABS, F32_REL_L2 = 1e-3, 1e-4
BF16_REL_L2 = 2e-2
# bf16 / 4-bit stages, every row by itself (a row = the last axis: one token's hidden state, or one cached key or
# value vector of one head): a whole-tensor norm over hundreds of rows would let a single wrong row through.
# Largest rows observed over all GPU parity tests: 2.2e-2 for a hidden-state row and 2.8e-2 for a cached key (layer 10
# of the 13B-shaped stage, a key of small norm: rounding noise grows with depth and is measured against the row's
# own norm); a row that is wrong in structure (a stale or misplaced tile, a wrong position) is off by tens of per cent.
BF16_ROW_REL_L2 = 4e-2


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def row_rel_l2(got, want):
    """Relative L2 error of every row (last axis) by itself; shape = got.shape[:-1].  Rows of the expected tensor
    that are (nearly) zero are measured against a hundredth of the mean row norm instead of their own."""
    g = np.asarray(got, dtype=np.float64)
    w = np.asarray(want, dtype=np.float64)
    den = np.linalg.norm(w, axis=-1)
    floor = 1e-2 * float(den.mean()) if den.size else 0.0
    return np.linalg.norm(g - w, axis=-1) / np.maximum(den, max(floor, 1e-300))


def assert_rows_close(got, want, bound=BF16_ROW_REL_L2, what=""):
    """Every row within `bound`; the message names the worst row."""
    got, want = np.asarray(got), np.asarray(want)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if got.size == 0:
        return 0.0
    err = row_rel_l2(got, want)
    worst = np.unravel_index(int(np.argmax(err)), err.shape) if err.ndim else ()
    assert float(err.max()) <= bound, (what, "worst row", tuple(int(i) for i in worst), float(err.max()),
                                       "rows above the bound", int((err > bound).sum()), "of", err.size)
    LAST_WORST[0] = (float(err.max()), what, tuple(int(i) for i in worst), tuple(got.shape))
    return float(err.max())


# largest per-row errors seen by Pair.check in this process, per dtype: (error, what, row index, tensor shape), for
# the summary line at the end of a test run
WORST_ROW = {}
LAST_WORST = [None]


def to_numpy(t):
    import torch
    return t.detach().to(torch.float32).cpu().numpy()


class Pair:
    """An oracle stage and a GPU stage built from the same seeded tensors."""

    def __init__(self, cfg, dtype, seed, max_positions, max_chunk_tokens, weight_std=0.02, layers_np=None,
                 oracle_positions=None, w4_expanded=False):
        import torch
        self.cfg, self.dtype, self.seed = dict(cfg), dtype, seed
        bf16 = dtype != "f32"
        if dtype == "w4":
            # 4-bit stage: the GPU gets codes and scales, the oracle the matrices they expand to
            from oracle import w4
            self.layers_np = layers_np if layers_np is not None else si.make_w4_layers(cfg, seed, weight_std=weight_std)
            self.oracle = oracle.OracleStage(cfg, w4.dequantize_layers(self.layers_np), oracle_positions or max_positions)
            dev_layers = jb.upload_w4_layers(self.layers_np)
        else:
            self.layers_np = layers_np if layers_np is not None else si.make_layers(cfg, seed, bf16=bf16,
                                                                                    weight_std=weight_std)
            self.oracle = oracle.OracleStage(cfg, self.layers_np, oracle_positions or max_positions)
            dev_layers = jb.upload_layers(self.layers_np, dtype)
        self.stage = jb.Stage(cfg, dtype, dev_layers, max_chunk_tokens, w4_expanded=w4_expanded)
        torch.cuda.synchronize()
        del dev_layers  # the stage keeps its own packed copy
        self.kv = jb.KvCache(cfg, dtype, max_positions)
        self.td = torch.float32 if dtype == "f32" else torch.bfloat16

    def hidden(self, n_tokens, tag=0):
        return si.make_hidden(self.cfg, self.seed, n_tokens, tag=tag, bf16=self.dtype != "f32")

    def gpu_chunk(self, hidden_np, pos, kv=None):
        import torch
        x = torch.from_numpy(hidden_np).to(device="cuda:0", dtype=self.td)
        y = self.stage.prefill_chunk(x, pos, kv if kv is not None else self.kv)
        torch.cuda.synchronize()
        return to_numpy(y)

    def gpu_tree(self, hidden_np, pos, parents, kv=None):
        import torch
        x = torch.from_numpy(hidden_np).to(device="cuda:0", dtype=self.td)
        y = self.stage.prefill_tree(x, pos, parents, kv if kv is not None else self.kv)
        torch.cuda.synchronize()
        return to_numpy(y)

    def run_both(self, hidden_np, chunks, reset=True):
        """Feeds the chunks to both sides; returns (gpu_out, oracle_out) concatenated over the chunks."""
        if reset:
            self.kv.reset()
            self.oracle.reset()
        g, o, p = [], [], len(self.kv)
        row = 0
        for n in chunks:
            h = hidden_np[row:row + n]
            g.append(self.gpu_chunk(h, p))
            o.append(self.oracle.prefill_chunk(h, p))
            p += n
            row += n
        return np.concatenate(g, axis=0), np.concatenate(o, axis=0)

    def kv_gpu(self):
        return to_numpy(self.kv.view())

    def check(self, got, want, what=""):
        if self.dtype == "f32":
            assert np.max(np.abs(got - want)) <= F32_MAX_ABS, (what, float(np.max(np.abs(got - want))))
            assert rel_l2(got, want) <= F32_REL_L2, (what, rel_l2(got, want))
        else:
            assert np.all(np.isfinite(got)), what
            assert rel_l2(got, want) <= BF16_REL_L2, (what, rel_l2(got, want))
            if np.ndim(got) >= 2:
                assert_rows_close(got, want, BF16_ROW_REL_L2, what)
                WORST_ROW.setdefault(self.dtype, []).append(LAST_WORST[0])
                WORST_ROW[self.dtype] = sorted(WORST_ROW[self.dtype], reverse=True)[:5]
