"""Pins of the oracle's reading of 4-bit weights (CPU only): the sixteen e2m1 code values and the
e8m0 scale as the open microscaling format defines them, written out by hand; nibble order; block
structure; exact representability of every product in bf16."""
from __future__ import annotations

import numpy as np

import oracle
import workloads as wl

# code -> value, by hand from the format's definition: 1 sign, 2 exponent (bias 1), 1 mantissa bit
E2M1_BY_HAND = {0b0000: 0.0, 0b0001: 0.5, 0b0010: 1.0, 0b0011: 1.5, 0b0100: 2.0, 0b0101: 3.0, 0b0110: 4.0, 0b0111: 6.0,
                0b1000: -0.0, 0b1001: -0.5, 0b1010: -1.0, 0b1011: -1.5, 0b1100: -2.0, 0b1101: -3.0, 0b1110: -4.0,
                0b1111: -6.0}


def test_every_code_and_the_scale_exponent():
    # 32 elements = one block: codes 0..15 twice; element with even k in the low nibble
    nibbles = np.array(list(range(16)) * 2, dtype=np.uint8)
    codes = (nibbles[0::2] | (nibbles[1::2] << 4)).astype(np.uint8)[None, :]
    for byte, scale in ((127, 1.0), (128, 2.0), (120, 2.0 ** -7), (119, 2.0 ** -8), (130, 8.0)):
        v = oracle.dequant_mxfp4(codes, np.array([[byte]], dtype=np.uint8))
        want = np.array([E2M1_BY_HAND[int(c)] * scale for c in nibbles])
        assert np.array_equal(v[0], want)
        assert np.array_equal(np.signbit(v[0]), np.signbit(want))


def test_exponent_formula_matches_the_bit_layout():
    # e2m1 from its fields: subnormal (exp field 0) = mantissa * 0.5; normal = (1 + m/2) * 2^(exp-1)
    for c in range(16):
        s, e, m = c >> 3, (c >> 1) & 3, c & 1
        val = (m * 0.5 if e == 0 else (1 + m / 2) * 2.0 ** (e - 1)) * (-1 if s else 1)
        assert val == E2M1_BY_HAND[c]


def test_each_block_of_32_has_its_own_scale_and_rows_are_independent():
    rng = np.random.default_rng(3)
    codes = rng.integers(0, 256, size=(3, 5, 48), dtype=np.uint8)          # K = 96 = 3 blocks
    scales = rng.integers(117, 131, size=(3, 5, 3), dtype=np.uint8)
    v = oracle.dequant_mxfp4(codes, scales)
    assert v.shape == (3, 5, 96)
    for (e, r, k) in [(0, 0, 0), (2, 4, 95), (1, 3, 31), (1, 3, 32), (0, 2, 63), (0, 2, 64)]:
        byte = codes[e, r, k // 2]
        nib = (byte >> 4) if k % 2 else (byte & 15)
        assert v[e, r, k] == E2M1_BY_HAND[int(nib)] * 2.0 ** (int(scales[e, r, k // 32]) - 127)


def test_synthetic_4bit_weights_are_exact_bf16_values_of_the_right_size():
    cfg = wl.LayerConfig("q", dtype="bf16", seed=12, E=3, k=2, H=128, F=192, N=8, n_ls=2, chunk_rows=8)
    w = wl.make_weights_mxfp4(cfg)
    assert w["W1q"].shape == (3, 192, 64) and w["W1s"].shape == (3, 192, 4)
    assert w["W2q"].shape == (3, 128, 96) and w["W2s"].shape == (3, 128, 6)
    wb = oracle.mxfp4_weights_as_bf16(w)                                   # asserts exactness itself
    for n in ("W1", "W3", "W2"):
        v = wl.as_f64(wb[n])
        assert np.array_equal(v, oracle.dequant_mxfp4(w[n + "q"], w[n + "s"]))
        assert 0.015 < v.std() < 0.04                                      # the scale of the bf16 recipe
        assert len(np.unique(w[n + "s"])) == 3 and len(np.unique(w[n + "q"])) == 256
