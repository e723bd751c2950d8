"""Pins of the 4-bit weight format the quantised stage reads (oracle side, CPU only).

The paper names INT4 (Sec. VI-A) without a scheme; the format is this build's own and these tests pin its
expansion to values worked out by hand, so that a swapped nibble, a wrong zero point or a transposed scale
fails here."""
import numpy as np

from oracle import w4
from paper_2504_08242_amd import synth_inputs as si


def test_nibble_order_zero_point_and_scale_groups_by_hand():
    # one output row, 256 inputs = two scale groups; bytes written by hand
    packed = np.zeros((1, 128), dtype=np.uint8)
    packed[0, 0] = 0x8F     # k = 0 -> code 15 (low nibble), k = 1 -> code 8 (high nibble)
    packed[0, 1] = 0x07     # k = 2 -> code 7, k = 3 -> code 0
    packed[0, 64] = 0x19    # k = 128 -> code 9, k = 129 -> code 1 (second group)
    scales = np.array([[0.5, 3.0]], dtype=np.float32)
    w = w4.dequantize(packed, scales)
    assert w.shape == (1, 256)
    assert w[0, 0] == 0.5 * 7 and w[0, 1] == 0.0 and w[0, 2] == -0.5 and w[0, 3] == -4.0
    assert w[0, 4] == -4.0                      # byte 0x00: code 0 -> -8 * 0.5
    assert w[0, 128] == 3.0 and w[0, 129] == -21.0
    assert w[0, 130] == -24.0


def test_scales_belong_to_rows_not_columns():
    packed = np.full((2, 64), 0x99, dtype=np.uint8)          # every code 9 -> +1
    scales = np.array([[2.0], [5.0]], dtype=np.float32)
    w = w4.dequantize(packed, scales)
    assert np.all(w[0] == 2.0) and np.all(w[1] == 5.0)


def test_unpack_is_the_inverse_of_packing_low_nibble_first():
    rng = np.random.default_rng(3)
    codes = rng.integers(0, 16, size=(5, 256), dtype=np.int32)
    packed = (codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8)
    assert np.array_equal(w4.unpack_codes(packed), codes)


def test_expansion_is_linear_in_the_scales_and_odd_in_the_codes():
    rng = np.random.default_rng(4)
    packed = rng.integers(0, 256, size=(3, 128), dtype=np.uint8)
    scales = rng.random((3, 2), dtype=np.float32) + 0.5
    w = w4.dequantize(packed, scales)
    assert np.array_equal(w4.dequantize(packed, 2 * scales), 2 * w)
    # code c -> 16 - c mirrors every level except -8 (code 0 has no partner)
    codes = w4.unpack_codes(packed)
    mirrored = np.where(codes == 0, 0, 16 - codes)
    mp = (mirrored[:, 0::2] | (mirrored[:, 1::2] << 4)).astype(np.uint8)
    wm = w4.dequantize(mp, scales)
    live = codes != 0
    assert np.array_equal(wm[live], -w[live])


def test_generated_layers_expand_to_weights_of_the_recipes_scale():
    cfg = dict(si.LLAMA7B_STAGE, n_layers=1, d_model=256, n_heads=2, d_ffn=384)
    layers = si.make_w4_layers(cfg, seed=5)
    assert layers[0]["wq"].shape == (256, 128) and layers[0]["wq"].dtype == np.uint8
    assert layers[0]["w_down"].shape == (256, 192) and layers[0]["w_down_scale"].shape == (256, 3)
    full = w4.dequantize_layers(layers)[0]
    assert full["w_gate"].shape == (384, 256)
    assert abs(float(np.std(full["w_up"])) - 0.02) < 0.003
    assert abs(float(np.mean(full["w_up"]))) < 1e-3
    # the same seed gives the same bytes; another layer index gives others
    again = si.make_w4_layers(cfg, seed=5)
    assert np.array_equal(again[0]["wo"], layers[0]["wo"])
