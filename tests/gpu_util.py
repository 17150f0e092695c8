"""Shared helpers of the GPU parity tests: build one problem for both sides.

Inputs come from keep_synth (seeded draws) and, for the group caches, from the CPU
oracle's own group-local prefill; nothing the oracle reads ever comes from the GPU.
"""
import numpy as np
import torch

import keep_synth as ks
from oracle import keep_oracle as ko
from oracle_util import layer_to_numpy, oracle_shape


def max_rel(a: np.ndarray, b: np.ndarray) -> float:
    """max |a - b| / max |b| (the tolerance metric of the parity tests)."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.abs(b).max()
    return float(np.abs(a - b).max() / (den if den > 0 else 1.0))


def mean_rel(a: np.ndarray, b: np.ndarray) -> float:
    """mean |a - b| / mean |b| (reported beside the maximum; not a tolerance)."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.abs(b).mean()
    return float(np.abs(a - b).mean() / (den if den > 0 else 1.0))


def update_err(x_out: np.ndarray, x_in: np.ndarray, ref_out: np.ndarray, storage: str):
    """Error of the layer's UPDATE (x_out - x_in: output projection of the attention plus FFN), relative to the
    largest reference update, and the share of that error the output format itself accounts for.

    The residual stream is several times larger than what a layer adds to it, so max|a-b| / max|b| over x_out
    would let an attention error of tens of percent through; the update has no such cushion.  x_out is stored
    in `storage`: writing it costs up to half an ulp of the largest output, 2^-9 max|x_out| in bf16
    (2^-25 in fp32), which the returned allowance expresses in units of the largest update.
    Returns (error, allowance): assert error < tol + allowance."""
    x_out, x_in, ref_out = (np.asarray(v, dtype=np.float64) for v in (x_out, x_in, ref_out))
    d_ref = ref_out - x_in
    den = max(np.abs(d_ref).max(), 1e-300)
    err = float(np.abs((x_out - x_in) - d_ref).max() / den)
    half_ulp = 2.0 ** -9 if storage == "bf16" else 2.0 ** -25
    return err, float(half_ulp * np.abs(ref_out).max() / den)


def layer_state_err(ctx, n_rows: int, probe: dict, lse_ref: np.ndarray, rows=None):
    """The attention output and the log-sum-exp that keep_recompute_layer left in the workspace against the
    oracle's (probe["attn_out"], lse_ref), each relative to its own largest value; `rows` restricts the
    device side to the rows the oracle evaluated.  Returns (attention error, log-sum-exp error)."""
    from paper_2602_23592_amd.binding import KEEP_STATE_ATTN_OUT, KEEP_STATE_LSE
    o = ctx.read_layer_state(KEEP_STATE_ATTN_OUT, n_rows).astype(np.float64)
    lse = ctx.read_layer_state(KEEP_STATE_LSE, n_rows).astype(np.float64)
    if rows is not None:
        o, lse = o[rows], lse[rows]
    return max_rel(o, probe["attn_out"]), max_rel(lse, lse_ref)


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float64).numpy()


class Problem:
    """Weights, prompt and oracle-made group caches on the host (f64) and on the GPU."""

    def __init__(self, shape: ks.ModelShape, group_len, instr_len, seed=0, std=0.05, bias=True, embed_scale=1.0,
                 random_cache=False, device="cuda"):
        self.shape = shape
        self.group_len = [int(v) for v in group_len]
        self.instr_len = int(instr_len)
        self.n_mem = sum(self.group_len)
        self.n_tokens = self.n_mem + self.instr_len
        dt = ks.torch_dtype(shape.storage)
        layers_t, embed_t = ks.make_weights(shape, "cpu", std=std, bias=bias, norm_jitter=0.1)
        embed_t = (embed_t.float() * (embed_scale / std)).to(dt)
        self.sh = oracle_shape(shape)
        self.layers = [layer_to_numpy(w) for w in layers_t]
        self.embed = ks.to_numpy_f64(embed_t)
        self.ids = ks.make_token_ids(self.n_tokens, shape.vocab, seed)
        if random_cache:
            self.kb, self.vb, kb_t, vb_t = [], [], [], []
            for l in range(shape.n_layers):
                k_t, v_t = ks.make_random_group_cache(shape, self.group_len, l, seed=seed + 7)
                kb_t.append(k_t); vb_t.append(v_t)
                self.kb.append([ks.to_numpy_f64(t) for t in k_t])
                self.vb.append([ks.to_numpy_f64(t) for t in v_t])
        else:
            self.kb, self.vb = ko.precompute_group_caches(self.sh, self.layers, self.embed, self.ids, self.group_len)
            kb_t = [[torch.from_numpy(b).to(dt) for b in row] for row in self.kb]
            vb_t = [[torch.from_numpy(b).to(dt) for b in row] for row in self.vb]
        # device side
        self.device = device
        self.layers_d = [{k: (None if v is None else v.to(device).contiguous()) for k, v in w.items()} for w in layers_t]
        self.embed_d = embed_t.to(device).contiguous()
        self.kb_d = [[t.to(device).contiguous() for t in row] for row in kb_t]
        self.vb_d = [[t.to(device).contiguous() for t in row] for row in vb_t]
        self.kb_t, self.vb_t = kb_t, vb_t

    def context(self, kernel_path=0, max_tokens=None, max_groups=None):
        from paper_2602_23592_amd import KeepContext
        return KeepContext(self.shape, self.layers_d, self.embed_d, max_tokens or self.n_tokens,
                           max_groups if max_groups is not None else max(1, len(self.group_len)), kernel_path)

    def prompt(self, pinned_host=False):
        from paper_2602_23592_amd import KeepPrompt
        from paper_2602_23592_amd.binding import KEEP_KV_DEVICE, KEEP_KV_PINNED_HOST
        if pinned_host:
            kb = [[t.contiguous().pin_memory() for t in row] for row in self.kb_t]
            vb = [[t.contiguous().pin_memory() for t in row] for row in self.vb_t]
            return KeepPrompt(self.group_len, self.instr_len, self.ids, kb, vb, self.shape.n_layers, KEEP_KV_PINNED_HOST)
        return KeepPrompt(self.group_len, self.instr_len, self.ids, self.kb_d, self.vb_d, self.shape.n_layers,
                          KEEP_KV_DEVICE)

    def empty_cache(self, n_layers=None):
        s = self.shape
        L = s.n_layers if n_layers is None else n_layers
        dt = ks.torch_dtype(s.storage)
        k = torch.full((L, self.n_tokens, s.n_kv_heads, s.head_dim), float("nan"), dtype=dt, device=self.device)
        return k, k.clone()

    def oracle_joined_cache(self, layer):
        return ko.realign_concat(self.sh, self.kb[layer], self.vb[layer], self.group_len, self.instr_len)
