"""Pins of the INT4 weight-only oracle (format of Section 6.1's weight-only quantisation): none of these
checks re-uses the oracle's own formula."""
import json
import os

import numpy as np
import torch

import keep_synth as ks
from oracle import int4_oracle as io

HERE = os.path.dirname(os.path.abspath(__file__))


def _fixture():
    with open(os.path.join(HERE, "golden", "int4_words.json")) as f:
        return json.load(f)


def test_nibble_order_against_hand_written_bytes():
    fx = _fixture()["nibble_order"]
    codes = np.zeros(32 * 128 // 2, dtype=np.uint8)                 # one block: 32 rows x 128 features
    codes[:8] = [int(h, 16) for h in fx["bytes_hex"]]               # first 8 bytes of row 0
    q = io.unpack_codes(codes, 32, 128)
    assert q[0, :16].tolist() == fx["codes"]
    assert not q[0, 16:].any() and not q[1:].any()


def test_block_addressing_against_hand_computed_offsets():
    ad = _fixture()["addressing"]
    rows, k = ad["rows"], ad["k"]
    for e in ad["code_at"]:
        codes = np.zeros(rows * k // 2, dtype=np.uint8)
        codes[e["byte"]] = 0xB0 if e["high"] else 0x0B
        q = io.unpack_codes(codes, rows, k)
        assert q[e["row"], e["feature"]] == 11, e
        assert np.count_nonzero(q) == 1, e
    one = int(ks.bf16_bits_from_f32(np.array([1.0], dtype=np.float32))[0])
    for e in ad["word_at"]:
        words = np.zeros(rows * k // 128, dtype=np.uint32)
        words[e["index"]] = one | (9 << 16)
        scale, zero = io.split_scale_zero(words, rows, k)
        assert scale[e["row"], e["group"]] == 1.0 and zero[e["row"], e["group"]] == 9, e
        assert np.count_nonzero(scale) == 1 and np.count_nonzero(zero) == 1, e


def test_scale_zero_word_and_weights_against_hand_computed_values():
    fx = _fixture()
    words = np.full(32, int(fx["scale_zero_hex"], 16), dtype=np.uint32)      # one block of 32 rows, one group
    scale, zero = io.split_scale_zero(words, 32, 128)
    assert scale[0, 0] == fx["scale"] and zero[0, 0] == fx["zero"]
    by = np.array([int(h, 16) for h in fx["nibble_order"]["bytes_hex"]], dtype=np.uint8)
    codes = np.tile(np.tile(by, 8), 32)                                      # every row: the 8 bytes, 8 times
    w = io.dequantize(codes, words, 32, 128)
    assert w.shape == (32, 128)
    assert w[0, :8].tolist() == fx["weights_first8"]
    assert np.array_equal(w[0, 16:24], w[0, :8]) and np.array_equal(w[17], w[0])


def test_generator_packing_is_the_documented_format():
    m = ks.make_int4_matrix(96, 384, seed=3)
    assert m["codes"].shape == (96 * 384 // 2,) and m["scale_zero"].shape == (96 * 3,)
    assert np.array_equal(io.unpack_codes(m["codes"], 96, 384), m["q"])
    scale, zero = io.split_scale_zero(m["scale_zero"], 96, 384)
    assert np.array_equal(zero, m["zero"].astype(np.int64))
    assert np.array_equal(scale, ks.f32_from_bf16_bits(m["scale_bits"]).astype(np.float64))


def test_rounding_is_round_to_nearest_even_like_torch():
    rng = np.random.default_rng(0)
    # products (q - z) * s with an 8-bit significand scale: the values the dequantiser rounds
    s = ks.f32_from_bf16_bits(ks.bf16_bits_from_f32(rng.uniform(1e-3, 0.1, size=4000).astype(np.float32))).astype(np.float64)
    d = rng.integers(-15, 16, size=4000).astype(np.float64)
    x = d * s
    want = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(io.round_to_bf16(x), want)
    # exact ties: 1 + 2^-8 (tie, even below) -> 1 ; 1 + 3 * 2^-8 (tie, odd below) -> 1 + 2^-6
    assert io.round_to_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert io.round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6


def test_closed_forms():
    rows, k = 64, 256
    q = (np.arange(rows * k, dtype=np.int64).reshape(rows, k) * 7 // 3 % 16).astype(np.uint8)
    codes = ks.pack_int4_codes(q)
    one = int(ks.bf16_bits_from_f32(np.array([1.0], dtype=np.float32))[0])
    ones = np.full((rows, k // 128), one, dtype=np.uint16)
    # scale 1, zero 0: the weights are the codes
    sz = ks.pack_int4_scale_zero(ones, np.zeros((rows, k // 128), dtype=np.uint8))
    assert np.array_equal(io.dequantize(codes, sz, rows, k), q.astype(np.float64))
    # zero point equal to every code: all weights 0
    q5 = np.full((rows, k), 5, dtype=np.uint8)
    sz5 = ks.pack_int4_scale_zero(ones, np.full((rows, k // 128), 5, dtype=np.uint8))
    assert not io.dequantize(ks.pack_int4_codes(q5), sz5, rows, k).any()
    # each (row, group) uses its own scale and zero
    half = int(ks.bf16_bits_from_f32(np.array([0.5], dtype=np.float32))[0])
    bits = np.tile(np.array([[one, half]], dtype=np.uint16), (rows, 1))
    bits[40, 1] = int(ks.bf16_bits_from_f32(np.array([2.0], dtype=np.float32))[0])
    zero = np.tile(np.array([[1, 2]], dtype=np.uint8), (rows, 1))
    zero[40, 1] = 3
    w = io.dequantize(codes, ks.pack_int4_scale_zero(bits, zero), rows, k)
    assert np.array_equal(w[:, :128], q[:, :128].astype(np.float64) - 1.0)
    keep = np.arange(rows) != 40
    assert np.array_equal(w[keep, 128:], (q[keep, 128:].astype(np.float64) - 2.0) * 0.5)
    assert np.array_equal(w[40, 128:], (q[40, 128:].astype(np.float64) - 3.0) * 2.0)


def test_matmul_with_dequantised_weights_against_integer_evaluation():
    """y = W x evaluated group by group in integers (sum of x * (q - z), then times the scale) agrees with the
    dequantised matrix wherever the product needs no rounding (power-of-two scales)."""
    rows, k = 32, 384
    rng = np.random.default_rng(2)
    q = rng.integers(0, 16, size=(rows, k)).astype(np.uint8)
    zero = rng.integers(0, 16, size=(rows, k // 128)).astype(np.uint8)
    expo = rng.integers(-9, -3, size=(rows, k // 128))
    bits = ks.bf16_bits_from_f32((2.0 ** expo).astype(np.float32))
    w = io.dequantize(ks.pack_int4_codes(q), ks.pack_int4_scale_zero(bits, zero), rows, k)
    x = rng.integers(-8, 9, size=k).astype(np.int64)
    want = np.zeros(rows)
    for r in range(rows):
        for g in range(k // 128):
            acc = 0
            for j in range(128 * g, 128 * (g + 1)):
                acc += int(x[j]) * (int(q[r, j]) - int(zero[r, g]))
            want[r] += acc * 2.0 ** int(expo[r, g])
    assert np.array_equal(w @ x.astype(np.float64), want)
