"""Seeded random draws and storage-format conversions (no method arithmetic)."""
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

from .configs import ModelShape, Workload


# ----------------------------------------------------------------------------
# storage-format conversion (IEEE binary32 <-> bfloat16 bit patterns)
# ----------------------------------------------------------------------------
def bf16_bits_from_f32(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even binary32 -> bfloat16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def f32_from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def torch_dtype(storage: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[storage]


def to_numpy_f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a stored tensor (fp32 or bf16) to float64 on the host."""
    return t.detach().to("cpu", torch.float64).numpy()


# ----------------------------------------------------------------------------
# group layout
# ----------------------------------------------------------------------------
def group_lengths(w: Workload, seed: int = 1) -> Tuple[np.ndarray, np.ndarray]:
    """Group lengths (int32) and kinds (uint8: 0 static, 1 dynamic) of a workload.

    Variable lengths are drawn uniformly in [lo, hi] from PCG64(seed); the last
    groups are then moved by +-1, staying in range, until the total is exact.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    lens: List[int] = []
    kinds: List[int] = []
    for count, lo, hi, kind in w.group_recipe:
        if lo == hi:
            lens += [lo] * count
        else:
            lens += [int(v) for v in rng.integers(lo, hi + 1, size=count)]
        kinds += [kind] * count
    lens_a = np.array(lens, dtype=np.int64)
    diff = int(w.mem_tokens - lens_a.sum())
    if diff != 0:
        # only variable-length recipes may be adjusted
        bounds = []
        for count, lo, hi, _ in w.group_recipe:
            bounds += [(lo, hi)] * count
        step = 1 if diff > 0 else -1
        i = len(lens_a) - 1
        guard = 0
        while diff != 0:
            lo, hi = bounds[i]
            if lo <= lens_a[i] + step <= hi:
                lens_a[i] += step
                diff -= step
            i = i - 1 if i > 0 else len(lens_a) - 1
            guard += 1
            if guard > 100 * len(lens_a) + abs(diff) * 4 + 1000000:
                raise ValueError("cannot reach the requested token total within the length range")
    assert int(lens_a.sum()) == w.mem_tokens
    return lens_a.astype(np.int32), np.array(kinds, dtype=np.uint8)


def make_token_ids(n_tokens: int, vocab: int, seed: int = 0) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(0, vocab, size=n_tokens, dtype=np.int64).astype(np.int32)


# ----------------------------------------------------------------------------
# weights
# ----------------------------------------------------------------------------
_LAYER_MATS = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown")


def layer_weight_shapes(s: ModelShape) -> Dict[str, Tuple[int, ...]]:
    """torch.nn.Linear layout: [out_features, in_features], row-major."""
    return {
        "ln1": (s.hidden,), "ln2": (s.hidden,),
        "wq": (s.q_dim, s.hidden), "wk": (s.kv_dim, s.hidden), "wv": (s.kv_dim, s.hidden),
        "wo": (s.hidden, s.q_dim),
        "wgate": (s.ffn_dim, s.hidden), "wup": (s.ffn_dim, s.hidden), "wdown": (s.hidden, s.ffn_dim),
    }


def make_layer_weights(s: ModelShape, layer: int, device: str = "cpu", std: float = 0.02,
                       bias: bool = False, norm_jitter: float = 0.0) -> Dict[str, torch.Tensor]:
    """One layer's weights, N(0, std) per matrix from torch.Generator(seed 1000+layer).

    RMSNorm weights are 1 (plus N(0, norm_jitter) when asked, so that tests can
    tell a dropped norm weight from a present one); QKV biases are absent unless
    `bias` (then N(0, std)).
    """
    g = torch.Generator(device=device)
    g.manual_seed(1000 + layer)
    dt = torch_dtype(s.storage)
    out: Dict[str, torch.Tensor] = {}
    shapes = layer_weight_shapes(s)
    for name in _LAYER_MATS:
        out[name] = (torch.randn(shapes[name], generator=g, device=device, dtype=torch.float32) * std).to(dt)
    for name in ("ln1", "ln2"):
        wln = torch.ones(shapes[name], device=device, dtype=torch.float32)
        if norm_jitter:
            wln = wln + torch.randn(shapes[name], generator=g, device=device, dtype=torch.float32) * norm_jitter
        out[name] = wln.to(dt)
    if bias:
        for name, n in (("bq", s.q_dim), ("bk", s.kv_dim), ("bv", s.kv_dim)):
            out[name] = (torch.randn((n,), generator=g, device=device, dtype=torch.float32) * std).to(dt)
    else:
        out["bq"] = out["bk"] = out["bv"] = None
    return out


def make_embedding(s: ModelShape, device: str = "cpu", std: float = 0.02, rows: Optional[int] = None) -> torch.Tensor:
    g = torch.Generator(device=device)
    g.manual_seed(999)
    n = s.vocab if rows is None else rows
    return (torch.randn((n, s.hidden), generator=g, device=device, dtype=torch.float32) * std).to(torch_dtype(s.storage))


def make_weights(s: ModelShape, device: str = "cpu", std: float = 0.02, bias: bool = False,
                 norm_jitter: float = 0.0):
    """(list of per-layer dicts, embedding table) in the storage dtype on `device`."""
    layers = [make_layer_weights(s, l, device, std, bias, norm_jitter) for l in range(s.n_layers)]
    return layers, make_embedding(s, device, std)


# ----------------------------------------------------------------------------
# INT4 weight-only matrices: random codes, zero points and scales (no dequantisation here)
# ----------------------------------------------------------------------------
INT4_GROUP = 128   # input features that share one scale and one zero point
INT4_MATS = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown")


INT4_ROWS = 32     # output rows per storage block


def pack_int4_codes(q: np.ndarray) -> np.ndarray:
    """Storage packing of 4-bit codes [rows, K] -> flat bytes [rows * K / 2].

    Blocks of 32 rows x 128 input features, ordered by (row block, feature group); inside a block the 32
    rows follow each other, 64 bytes each; within each run of 8 consecutive input features of a row, byte t
    (t < 4) holds feature t in its low nibble and feature t + 4 in its high nibble."""
    rows, k = q.shape
    assert rows % INT4_ROWS == 0 and k % INT4_GROUP == 0
    q8 = q.reshape(rows, k // 8, 8).astype(np.uint8)
    by = (q8[:, :, 0:4] | (q8[:, :, 4:8] << np.uint8(4))).reshape(rows // INT4_ROWS, INT4_ROWS, k // INT4_GROUP, 64)
    return np.ascontiguousarray(by.transpose(0, 2, 1, 3)).reshape(-1)


def pack_int4_scale_zero(scale_bits: np.ndarray, zero: np.ndarray) -> np.ndarray:
    """[rows, K/128] scale patterns and zero points -> flat uint32 words in block order (32 words per block)."""
    rows, kg = scale_bits.shape
    w = scale_bits.astype(np.uint32) | (zero.astype(np.uint32) << np.uint32(16))
    return np.ascontiguousarray(w.reshape(rows // INT4_ROWS, INT4_ROWS, kg).transpose(0, 2, 1)).reshape(-1)


def make_int4_matrix(rows: int, k: int, seed: int, std: float = 0.02) -> Dict[str, np.ndarray]:
    """Random group-quantised matrix: codes ~ Binomial(15, 1/2), zero point 7 or 8, bf16 scale drawn so
    that (code - zero) * scale has a standard deviation near `std`.

    Returns the raw draws (`q` [rows, K] uint8, `zero` [rows, K/128] uint8, `scale_bits` [rows, K/128]
    uint16 bf16 patterns) and their storage form: `codes` (pack_int4_codes) and `scale_zero`
    (pack_int4_scale_zero), plus `rows` and `k`."""
    assert k % INT4_GROUP == 0 and rows % INT4_ROWS == 0
    rng = np.random.Generator(np.random.PCG64(seed))
    q = rng.binomial(15, 0.5, size=(rows, k)).astype(np.uint8)
    zero = rng.integers(7, 9, size=(rows, k // INT4_GROUP)).astype(np.uint8)
    scale = (std / 1.94) * rng.uniform(0.75, 1.25, size=(rows, k // INT4_GROUP))
    scale_bits = bf16_bits_from_f32(scale.astype(np.float32))
    return {"q": q, "zero": zero, "scale_bits": scale_bits, "codes": pack_int4_codes(q),
            "scale_zero": pack_int4_scale_zero(scale_bits, zero), "rows": rows, "k": k}


def make_int4_layer(s: ModelShape, layer: int, std: float = 0.02) -> Dict[str, Dict[str, np.ndarray]]:
    """The seven projection matrices of one layer as random INT4 matrices (seed 5000 + 16 * layer + index)."""
    shapes = layer_weight_shapes(s)
    return {name: make_int4_matrix(shapes[name][0], shapes[name][1], 5000 + 16 * layer + i, std)
            for i, name in enumerate(INT4_MATS)}


def make_int4_layer_on_device(s: ModelShape, layer: int, device: str = "cuda", std: float = 0.02):
    """Full-size stand-in drawn on the device (the numpy draws above take minutes at 14B/32B shapes):
    uniform code bytes, zero point 7 or 8, bf16 scale std / 4.6 * U[0.75, 1.25] (uniform codes have a
    standard deviation of 4.6); independent draws, so the storage order needs no permutation.
    Returns name -> (codes uint8 [rows * K / 2], scale_zero int32 [rows * K / 128], rows, K)."""
    g = torch.Generator(device=device)
    g.manual_seed(7000 + layer)
    shapes = layer_weight_shapes(s)
    out = {}
    for name in INT4_MATS:
        rows, k = shapes[name]
        codes = torch.randint(0, 256, (rows * k // 2,), generator=g, device=device, dtype=torch.uint8)
        zero = torch.randint(7, 9, (rows * k // INT4_GROUP,), generator=g, device=device, dtype=torch.int32)
        scale = (std / 4.6) * (0.75 + 0.5 * torch.rand((rows * k // INT4_GROUP,), generator=g, device=device))
        bits = scale.to(torch.bfloat16).view(torch.int16).to(torch.int32) & 0xFFFF
        out[name] = (codes, (bits | (zero << 16)).contiguous(), rows, k)
    return out


# ----------------------------------------------------------------------------
# random stand-ins for cached K/V blocks and hidden rows (teacher-forced layer tests)
# ----------------------------------------------------------------------------
def make_random_group_cache(s: ModelShape, group_len: Sequence[int], layer: int, seed: int = 7,
                            device: str = "cpu", std: float = 1.0):
    """Per-group K and V blocks [len_g, n_kv_heads, head_dim] of one layer, N(0, std)."""
    g = torch.Generator(device=device)
    g.manual_seed(seed * 100003 + layer)
    dt = torch_dtype(s.storage)
    ks, vs = [], []
    for n in group_len:
        ks.append((torch.randn((int(n), s.n_kv_heads, s.head_dim), generator=g, device=device) * std).to(dt))
        vs.append((torch.randn((int(n), s.n_kv_heads, s.head_dim), generator=g, device=device) * std).to(dt))
    return ks, vs


def make_random_rows(n: int, d: int, storage: str, seed: int = 11, device: str = "cpu", std: float = 1.0):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return (torch.randn((n, d), generator=g, device=device) * std).to(torch_dtype(storage))
