"""CPU oracle of the INT4 weight-only format (Section 6.1 runs the 32B model with INT4 weight-only
quantisation in the manner of AWQ: 4-bit codes, one scale and one zero point per group of input features).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the bench's CPU leg may use it; the product path
never does.  Plain numpy, written from the format's definition:

  * a matrix W[out, in] is stored as 4-bit codes q, and per (output row, group of 128 consecutive
    input features) a bfloat16 scale s and a 4-bit zero point z;
  * the weight the model computes with is  w = bf16( (q - z) * s ),  rounded to nearest even;
    (q - z) * s has at most 13 significant bits, so the product itself is exact in binary32 and
    the only rounding is the final one to bfloat16;
  * storage: codes packed two per byte, [out, in/2]: within each run of 8 consecutive input features
    byte t (t < 4) carries feature t in its low nibble and feature t + 4 in its high nibble;
    scale and zero point share one 32-bit word per (row, group): bits 0..15 the scale's bfloat16
    pattern, bits 16..19 the zero point, the rest 0.

Readings (the paper only names the scheme): group length 128 and asymmetric zero points as in the
cited scheme's usual configuration; the calibration that chooses codes and scales is outside this
build (weights arrive quantised).

Pins (tests/test_int4_oracle.py): the unpacking order against a hand-written byte fixture
(tests/golden/int4_words.json), the rounding against torch's float32 -> bfloat16 conversion, closed
forms (zero point = code -> 0; scale 1, zero 0 -> the code itself), and a matmul with dequantised
weights against an integer-arithmetic evaluation of sum a * (q - z) per group times the scale.
"""
import numpy as np

GROUP = 128


def unpack_codes(codes: np.ndarray) -> np.ndarray:
    """bytes [rows, K/2] -> codes [rows, K] (uint8 in 0..15)."""
    rows, half = codes.shape
    b = np.asarray(codes, dtype=np.uint8).reshape(rows, half // 4, 4)
    q = np.empty((rows, half // 4, 8), dtype=np.uint8)
    for t in range(4):
        q[:, :, t] = b[:, :, t] & 0x0F          # feature t of the run of eight
        q[:, :, t + 4] = b[:, :, t] >> 4        # feature t + 4
    return q.reshape(rows, half * 2)


def split_scale_zero(scale_zero: np.ndarray):
    """uint32 words -> (scale as float64, exactly the bfloat16 value; zero point as int)."""
    w = np.asarray(scale_zero, dtype=np.uint32)
    scale = ((w & np.uint32(0xFFFF)) << np.uint32(16)).view(np.float32).astype(np.float64)
    zero = ((w >> np.uint32(16)) & np.uint32(0xF)).astype(np.int64)
    return scale, zero


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even to bfloat16 of values exactly representable in binary32; float64 out."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    assert np.array_equal(f.astype(np.float64), np.asarray(x, dtype=np.float64)), "value not exact in binary32"
    u = f.view(np.uint32).astype(np.uint64)
    low = u & np.uint64(0xFFFF)
    up = u >> np.uint64(16)
    round_up = (low > 0x8000) | ((low == 0x8000) & ((up & np.uint64(1)) == 1))
    up = up + round_up.astype(np.uint64)
    return (up.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def dequantize(codes: np.ndarray, scale_zero: np.ndarray) -> np.ndarray:
    """The weights the model computes with, [rows, K] float64 (each value a bfloat16 number)."""
    q = unpack_codes(codes).astype(np.int64)
    scale, zero = split_scale_zero(scale_zero)
    rows, k = q.shape
    assert scale.shape == (rows, k // GROUP)
    diff = q.reshape(rows, k // GROUP, GROUP) - zero[:, :, None]
    return round_to_bf16(diff.astype(np.float64) * scale[:, :, None]).reshape(rows, k)
