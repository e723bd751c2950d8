"""Plain definition of a stage forward over a WHOLE prompt -- TEST INFRASTRUCTURE.

The chunk-by-chunk method of Sec. IV-A.2 of the Jupiter paper reaches exactly
(up to rounding order) what a causal decoder computes on the whole prompt at
once; this file writes that definition out in numpy fp64: no KV cache, no
sub-sequences, an explicit S x S score matrix with an explicit mask, softmax
over whole rows.  The decoder layer is that of Sec. II-A in the Llama-2 form
(pre-norm RMSNorm, half-split rotary embedding, SwiGLU, no bias).

It serves as the brute-force pin of ``jupiter_oracle.c`` and is itself pinned
against library routines in ``tests/``.  Nothing outside ``tests/``, the smoke
check and the benchmark's CPU-baseline leg may import it, and it imports
nothing from the HIP path.
"""
import numpy as np

WEIGHT_NAMES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "g_attn", "g_mlp")


def rmsnorm(x, g, eps):
    """Row-wise x * g / sqrt(mean(x^2) + eps)."""
    x = np.asarray(x, dtype=np.float64)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * np.asarray(g, dtype=np.float64)


def rope(x, positions, theta):
    """Rotate pairs (i, i + dh/2) of x[..., S, dh] by positions[s] * theta**(-2i/dh)."""
    x = np.asarray(x, dtype=np.float64)
    dh = x.shape[-1]
    half = dh // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / dh)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]
    c, s = np.cos(ang), np.sin(ang)
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(z):
    return z / (1.0 + np.exp(-z))


def causal_attention(q, k, v):
    """q, k, v: [H, S, dh]; query s sees keys 0..s (itself included)."""
    H, S, dh = q.shape
    scores = np.einsum("hsd,htd->hst", q, k) / np.sqrt(float(dh))
    masked = np.triu(np.ones((S, S), dtype=bool), k=1)  # key index > query index
    scores = np.where(masked[None], -np.inf, scores)
    scores = scores - scores.max(axis=-1, keepdims=True)
    p = np.exp(scores)
    p = p / p.sum(axis=-1, keepdims=True)
    return np.einsum("hst,htd->hsd", p, v)


def stage_full(cfg, layers, hidden):
    """Forward of all layers over the whole prompt.

    cfg: dict with n_heads, head_dim, rms_eps, rope_theta.
    layers: list of dicts keyed by WEIGHT_NAMES (matrices [out, in]).
    hidden: [S, d].
    Returns (hidden_out [S, d], k [L, H, S, dh] after RoPE, v [L, H, S, dh]).
    """
    H, dh = cfg["n_heads"], cfg["head_dim"]
    x = np.asarray(hidden, dtype=np.float64)
    S = x.shape[0]
    pos = np.arange(S)
    ks, vs = [], []
    for w in layers:
        w = {n: np.asarray(w[n], dtype=np.float64) for n in WEIGHT_NAMES}
        xn = rmsnorm(x, w["g_attn"], cfg["rms_eps"])
        q = (xn @ w["wq"].T).reshape(S, H, dh).transpose(1, 0, 2)
        k = (xn @ w["wk"].T).reshape(S, H, dh).transpose(1, 0, 2)
        v = (xn @ w["wv"].T).reshape(S, H, dh).transpose(1, 0, 2)
        q = rope(q, pos, cfg["rope_theta"])
        k = rope(k, pos, cfg["rope_theta"])
        ks.append(k)
        vs.append(v)
        o = causal_attention(q, k, v).transpose(1, 0, 2).reshape(S, H * dh)
        h = x + o @ w["wo"].T
        hn = rmsnorm(h, w["g_mlp"], cfg["rms_eps"])
        x = h + (silu(hn @ w["w_gate"].T) * (hn @ w["w_up"].T)) @ w["w_down"].T
    return x, np.stack(ks) if ks else np.zeros((0, H, S, dh)), np.stack(vs) if vs else np.zeros((0, H, S, dh))
