"""Workload shapes: random-init Qwen-shaped decoders and memory-group layouts.

The paper measures on embodied-planning prompts (retrieved memory groups
followed by an instruction, Section 1 and Section 6.1) that are not available
here; these seeded synthetic shapes stand in for them.  A workload is only a
description: sizes, group-length recipe, recompute ratio and hop count.
"""
from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn_dim: int
    vocab: int
    rope_theta: float = 1.0e6
    rms_eps: float = 1.0e-6
    storage: str = "bf16"          # "f32" or "bf16": dtype of weights, caches, activations in HBM

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim


@dataclass(frozen=True)
class Workload:
    name: str
    shape: ModelShape
    # list of (count, lo, hi, kind): `count` groups with lengths uniform in [lo, hi]
    # (lo == hi: fixed length); kind 0 = static group, 1 = dynamic segment.
    group_recipe: Tuple[Tuple[int, int, int, int], ...]
    mem_tokens: int                 # exact sum of group lengths
    instr_len: int
    ratio: float                    # mean recompute ratio over layers 1..L-1
    hops: int
    kv_location: str = "device"     # "device" or "pinned_host"
    schedule: str = "linear"
    # what the ratio counts: "groups" (share of the memories) or "tokens" (share of the memory
    # tokens; used where group sizes differ by an order of magnitude, so that the ratio still
    # bounds the recomputed rows)
    budget: str = "groups"


_TINY = ModelShape(2, 256, 4, 2, 64, 688, 4096, storage="f32")
_Q7B = ModelShape(28, 3584, 28, 4, 128, 18944, 152064)
_Q14B = ModelShape(48, 5120, 40, 8, 128, 13824, 152064)
_Q32B = ModelShape(64, 5120, 40, 8, 128, 27648, 152064)

WORKLOADS = {
    "tiny": Workload("tiny", _TINY, ((8, 128, 128, 1),), 1024, 64, 0.15, 1),
    "qwen7b_16k": Workload("qwen7b_16k", _Q7B, ((64, 256, 256, 1),), 16384, 256, 0.15, 2),
    "qwen14b_32k": Workload("qwen14b_32k", _Q14B, ((16, 1024, 1024, 0), (256, 64, 64, 1)),
                            32768, 256, 0.10, 3, budget="tokens"),
    "qwen32b_32k_host": Workload("qwen32b_32k_host", _Q32B, ((128, 128, 384, 1),), 32768, 256,
                                 0.10, 2, kv_location="pinned_host"),
    "qwen14b_64k_stress": Workload("qwen14b_64k_stress", _Q14B, ((1024, 32, 96, 1),), 65536, 256,
                                   0.10, 3),
}


def workload(name: str) -> Workload:
    return WORKLOADS[name]


def ratio_schedule(ratio: float, n_layers: int, kind: str = "linear") -> np.ndarray:
    """Per-layer recompute ratios as float32: layer 0 recomputes everything
    (Section 4.2, last paragraph), later layers decrease.

    "linear": 1.5*ratio at layer 1 falling to 0.5*ratio at the last layer
    (mean `ratio` over layers 1..L-1).  "const": `ratio` at every layer >= 1.
    """
    r = np.empty(n_layers, dtype=np.float32)
    r[0] = 1.0
    for l in range(1, n_layers):
        if kind == "const" or n_layers <= 2:
            r[l] = ratio
        elif kind == "linear":
            r[l] = ratio * (1.5 - (l - 1) / (n_layers - 2))
        else:
            raise ValueError(kind)
    return r
