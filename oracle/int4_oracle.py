"""CPU oracle of the INT4 weight-only format (Section 6.1 runs the 32B model with INT4 weight-only
quantisation in the manner of AWQ: 4-bit codes, one scale and one zero point per group of input features).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the bench's CPU leg may use it; the product path
never does.  Plain numpy, written from the format's definition:

  * a matrix W[out, in] is stored as 4-bit codes q, and per (output row, group of 128 consecutive
    input features) a bfloat16 scale s and a 4-bit zero point z;
  * the weight the model computes with is  w = bf16( (q - z) * s ),  rounded to nearest even;
    (q - z) * s has at most 13 significant bits, so the product itself is exact in binary32 and
    the only rounding is the final one to bfloat16;
  * storage (rows a multiple of 32): codes packed two per byte in blocks of 32 rows x 128 input
    features, blocks ordered by (row block, feature group), 2048 bytes each; inside a block the 32 rows
    follow each other, 64 bytes per row; within each run of 8 consecutive input features byte t (t < 4)
    carries feature t in its low nibble and feature t + 4 in its high nibble;
    scale and zero point share one 32-bit word per (row, group): bits 0..15 the scale's bfloat16
    pattern, bits 16..19 the zero point, the rest 0; the words are stored in the same block order,
    32 words (one per row) per block.

Readings (the paper only names the scheme): group length 128 and asymmetric zero points as in the
cited scheme's usual configuration; the calibration that chooses codes and scales is outside this
build (weights arrive quantised).

Pins (tests/test_int4_oracle.py): the nibble order against hand-written bytes and the block
addressing against hand-computed byte offsets and word indices (tests/golden/int4_words.json), the rounding against torch's float32 -> bfloat16 conversion, closed
forms (zero point = code -> 0; scale 1, zero 0 -> the code itself), and a matmul with dequantised
weights against an integer-arithmetic evaluation of sum a * (q - z) per group times the scale.
"""
import numpy as np

GROUP = 128


ROWS = 32


def unpack_codes(codes: np.ndarray, rows: int, k: int) -> np.ndarray:
    """flat storage bytes -> codes [rows, K] (uint8 in 0..15)."""
    by = np.asarray(codes, dtype=np.uint8).reshape(rows // ROWS, k // GROUP, ROWS, 64)   # (row block, group, row, byte)
    q = np.empty((rows, k), dtype=np.uint8)
    for rb in range(rows // ROWS):
        for kg in range(k // GROUP):
            blk = by[rb, kg]                                   # [32 rows, 64 bytes]
            for run in range(GROUP // 8):
                for t in range(4):
                    b = blk[:, 4 * run + t]
                    q[rb * ROWS:(rb + 1) * ROWS, kg * GROUP + 8 * run + t] = b & 0x0F          # feature t of the run
                    q[rb * ROWS:(rb + 1) * ROWS, kg * GROUP + 8 * run + t + 4] = b >> 4        # feature t + 4
    return q


def split_scale_zero(scale_zero: np.ndarray, rows: int, k: int):
    """flat storage words -> (scale [rows, K/128] as float64, exactly the bfloat16 value; zero point as int)."""
    w = np.asarray(scale_zero, dtype=np.uint32).reshape(rows // ROWS, k // GROUP, ROWS)
    w = w.transpose(0, 2, 1).reshape(rows, k // GROUP)
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


def dequantize(codes: np.ndarray, scale_zero: np.ndarray, rows: int, k: int) -> np.ndarray:
    """The weights the model computes with, [rows, K] float64 (each value a bfloat16 number)."""
    q = unpack_codes(codes, rows, k).astype(np.int64)
    scale, zero = split_scale_zero(scale_zero, rows, k)
    diff = q.reshape(rows, k // GROUP, GROUP) - zero[:, :, None]
    return round_to_bf16(diff.astype(np.float64) * scale[:, :, None]).reshape(rows, k)
