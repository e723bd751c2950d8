"""4-bit weight format of the quantised stage -- TEST INFRASTRUCTURE (oracle side).

The paper runs both Llama-2 models with INT4 weights (Sec. VI-A) and names no quantisation scheme, so the
format is this build's own; it is the common group-wise symmetric one:

* a projection matrix W [out, in] is stored as 4-bit codes c in 0..15 and fp32 scales s [out, in / 128];
* W[n][k] = s[n][k // 128] * (c[n][k] - 8): sixteen levels -8..7 around zero, one scale per run of 128
  consecutive input features of an output row;
* the codes travel two per byte, row-major [out, in / 2]: byte j of a row holds c[2j] in its low four bits and
  c[2j + 1] in its high four bits.

The oracle of a quantised stage is the ordinary oracle stage run on the matrices this module expands; the
quantised arithmetic has no other definition.  RMSNorm gains, activations and the KV cache are not quantised.
"""
import numpy as np

GROUP = 128
MATRIX_NAMES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


def unpack_codes(packed):
    """uint8 [out, in/2] -> integer codes [out, in] (low nibble first)."""
    packed = np.asarray(packed, dtype=np.uint8)
    out = np.empty(packed.shape[:-1] + (packed.shape[-1] * 2,), dtype=np.int32)
    out[..., 0::2] = packed & 0x0F
    out[..., 1::2] = packed >> 4
    return out


def dequantize(packed, scales):
    """fp32 matrix [out, in] of a (packed codes, scales) pair."""
    codes = unpack_codes(packed)
    scales = np.asarray(scales, dtype=np.float32)
    n_out, n_in = codes.shape
    assert n_in % GROUP == 0 and scales.shape == (n_out, n_in // GROUP), (codes.shape, scales.shape)
    per_element = np.repeat(scales.astype(np.float64), GROUP, axis=1)
    return (per_element * (codes - 8)).astype(np.float32)


def dequantize_layers(layers_w4):
    """Layer dicts holding (name, name + '_scale') pairs and the two gains -> ordinary fp32 layer dicts."""
    out = []
    for w in layers_w4:
        d = {n: dequantize(w[n], w[n + "_scale"]) for n in MATRIX_NAMES}
        d["g_attn"], d["g_mlp"] = w["g_attn"], w["g_mlp"]
        out.append(d)
    return out
