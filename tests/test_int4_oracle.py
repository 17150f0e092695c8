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


def test_unpacking_order_against_hand_written_bytes():
    fx = _fixture()
    by = np.array([int(h, 16) for h in fx["bytes_hex"]], dtype=np.uint8).reshape(1, -1)
    assert io.unpack_codes(by).tolist() == [fx["codes"]]
    # two rows, the second with the runs swapped: rows and runs stay apart
    two = np.stack([by[0], np.concatenate([by[0, 4:], by[0, :4]])])
    got = io.unpack_codes(two)
    assert got[1].tolist() == fx["codes"][8:] + fx["codes"][:8]


def test_scale_zero_word_and_weights_against_hand_computed_values():
    fx = _fixture()
    word = np.array([[int(fx["scale_zero_hex"], 16)]], dtype=np.uint32)
    scale, zero = io.split_scale_zero(word)
    assert scale[0, 0] == fx["scale"] and zero[0, 0] == fx["zero"]
    by = np.array([int(h, 16) for h in fx["bytes_hex"]], dtype=np.uint8)
    codes = np.tile(by, 8).reshape(1, 64)                      # one group of 128 features
    w = io.dequantize(codes, word)
    assert w.shape == (1, 128)
    assert w[0, :8].tolist() == fx["weights_first8"]
    assert np.array_equal(w[0, 16:24], w[0, :8])


def test_generator_packing_is_the_documented_format():
    m = ks.make_int4_matrix(6, 256, seed=3)
    assert np.array_equal(io.unpack_codes(m["codes"]), m["q"])
    scale, zero = io.split_scale_zero(m["scale_zero"])
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
    rows, k = 3, 256
    q = np.arange(rows * k, dtype=np.uint8).reshape(rows, k) % 16
    codes = ks.pack_int4_codes(q)
    one = int(ks.bf16_bits_from_f32(np.array([1.0], dtype=np.float32))[0])
    # scale 1, zero 0: the weights are the codes
    sz = np.full((rows, k // 128), one, dtype=np.uint32)
    assert np.array_equal(io.dequantize(codes, sz), q.astype(np.float64))
    # zero point equal to every code: all weights 0
    q5 = np.full((rows, k), 5, dtype=np.uint8)
    sz5 = np.full((rows, k // 128), one | (5 << 16), dtype=np.uint32)
    assert not io.dequantize(ks.pack_int4_codes(q5), sz5).any()
    # each group uses its own scale and zero
    half = int(ks.bf16_bits_from_f32(np.array([0.5], dtype=np.float32))[0])
    szm = np.array([[one | (1 << 16), half | (2 << 16)]] * rows, dtype=np.uint32)
    w = io.dequantize(codes, szm)
    assert np.array_equal(w[:, :128], q[:, :128].astype(np.float64) - 1.0)
    assert np.array_equal(w[:, 128:], (q[:, 128:].astype(np.float64) - 2.0) * 0.5)


def test_matmul_with_dequantised_weights_against_integer_evaluation():
    """y = W x evaluated group by group in integers (sum of x * (q - z), then times the scale) agrees with the
    dequantised matrix wherever the product needs no rounding (power-of-two scales)."""
    rows, k = 5, 384
    rng = np.random.default_rng(2)
    q = rng.integers(0, 16, size=(rows, k)).astype(np.uint8)
    zero = rng.integers(0, 16, size=(rows, k // 128))
    expo = rng.integers(-9, -3, size=(rows, k // 128))
    bits = ks.bf16_bits_from_f32((2.0 ** expo).astype(np.float32)).astype(np.uint32)
    w = io.dequantize(ks.pack_int4_codes(q), bits | (zero.astype(np.uint32) << 16))
    x = rng.integers(-8, 9, size=k).astype(np.int64)
    want = np.zeros(rows)
    for r in range(rows):
        for g in range(k // 128):
            acc = 0
            for j in range(128 * g, 128 * (g + 1)):
                acc += int(x[j]) * (int(q[r, j]) - int(zero[r, g]))
            want[r] += acc * 2.0 ** int(expo[r, g])
    assert np.array_equal(w @ x.astype(np.float64), want)
