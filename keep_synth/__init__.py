"""Seeded synthetic inputs for the selective-KV-recompute prefill path.

This package is the only code shared by the CPU oracle's tests and the HIP
path's tests/bench.  It holds workload shapes and random-number recipes and
none of the method's arithmetic (no RoPE, no attention, no projections, no
selection): every array it returns is a plain random draw, a reshaping of
one, or a storage-format conversion (fp32 <-> bf16 bit patterns, 4-bit codes <-> packed bytes).
"""
from .configs import ModelShape, Workload, WORKLOADS, workload, ratio_schedule
from .gen import (
    bf16_bits_from_f32,
    f32_from_bf16_bits,
    torch_dtype,
    to_numpy_f64,
    group_lengths,
    layer_weight_shapes,
    make_layer_weights,
    make_embedding,
    make_weights,
    make_token_ids,
    make_random_group_cache,
    make_random_rows,
    INT4_GROUP,
    INT4_ROWS,
    INT4_MATS,
    pack_int4_codes,
    pack_int4_scale_zero,
    make_int4_matrix,
    make_int4_layer,
    make_int4_layer_on_device,
)
