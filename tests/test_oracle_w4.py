"""Pins for the 4-bit group weight storage (W4A16, the 13B setting of Sec. IV-A): the oracle's expansion to plain
weights against hand-written values, and the seeded quantiser's error bound."""
import numpy as np

from oracle import oracle
from paper_2507_02620_amd import synth


def test_dequant_hand_example():
    # one row, two groups of 128 columns; byte k//2 holds column k (even) in its low nibble
    codes = np.full((1, 128), 0x88, dtype=np.uint8)        # every code 8 -> weight 0
    codes[0, 0] = 0xF0                                      # column 0: code 0 -> -8 s, column 1: code 15 -> +7 s
    codes[0, 64] = 0x3A                                     # column 128: code 10 -> +2 s', column 129: code 3 -> -5 s'
    scales = np.array([[0.5, 0.25]], dtype=np.float32)
    w = oracle.dequant_w4(codes, scales)
    assert w.shape == (1, 256) and w.dtype == np.float32
    want = np.zeros(256, dtype=np.float32)
    want[0], want[1], want[128], want[129] = -4.0, 3.5, 0.5, -1.25
    assert np.array_equal(w[0], want)


def test_quantiser_error_bound_and_layout():
    w = synth.normal(3, 999, (48, 384), 0.02)
    codes, scales = synth.quantize_w4(w)
    assert codes.shape == (48, 192) and codes.dtype == np.uint8 and scales.shape == (48, 3)
    assert np.array_equal(scales, synth.round_bf16(scales))               # scales are bf16 values
    back = oracle.dequant_w4(codes, scales)
    err = np.abs(back - w).reshape(48, 3, 128)
    # nearest code within the range [-8, 7]: half a step, plus the rounding of the scale itself at the +7 end
    assert (err <= scales[:, :, None] * 0.5 * (1 + 2.0 ** -6)).all()
    # an independent per-element expansion
    rng = np.random.default_rng(0)
    for _ in range(200):
        n, k = int(rng.integers(48)), int(rng.integers(384))
        b = int(codes[n, k // 2])
        c = (b >> 4) if k & 1 else (b & 15)
        assert back[n, k] == np.float32(scales[n, k // 128]) * np.float32(c - 8)


def test_dequant_layer_keeps_other_tensors():
    cfg = synth.CONFIGS["C1"].with_(dtype="bf16", d_model=256, d_ffn=384)
    lw = synth.layer_weights_w4(cfg, 0, 1)
    plain = oracle.dequant_layer(lw)
    assert set(plain) == set(synth.layer_weights(cfg, 0, 1))
    assert plain["wq"].shape == (256, 256) and plain["w_down"].shape == (256, 384)
    assert np.array_equal(plain["rms_attn"], lw["rms_attn"])
    # the 4-bit matrices stay close to the matrices they were made from
    ref = synth.layer_weights(cfg, 0, 1)
    assert np.abs(plain["w_up"] - ref["w_up"]).max() < 0.02 * 4 / 7
