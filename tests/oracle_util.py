"""Helpers for tests that drive the CPU oracle (host side only)."""
import numpy as np

import keep_synth as ks
from oracle import keep_oracle as ko


def oracle_shape(s: ks.ModelShape, storage=None) -> ko.Shape:
    return ko.Shape(s.n_layers, s.hidden, s.n_q_heads, s.n_kv_heads, s.head_dim, s.ffn_dim, s.vocab,
                    s.rope_theta, s.rms_eps, storage or s.storage)


def layer_to_numpy(w: dict) -> dict:
    return {k: (None if v is None else ks.to_numpy_f64(v)) for k, v in w.items()}


def small_shape(storage="f64", **kw) -> ks.ModelShape:
    base = dict(n_layers=2, hidden=64, n_q_heads=4, n_kv_heads=2, head_dim=16, ffn_dim=96, vocab=97,
                rope_theta=1.0e4, rms_eps=1.0e-6, storage="f32")
    base.update(kw)
    return ks.ModelShape(**base)


def small_problem(shape: ks.ModelShape, group_len, instr_len, seed=0, std=0.2, bias=True, oracle_storage="f64"):
    """Weights (numpy f64), embedding, token ids and oracle-precomputed group caches."""
    layers_t, embed_t = ks.make_weights(shape, "cpu", std=std, bias=bias, norm_jitter=0.1)
    layers = [layer_to_numpy(w) for w in layers_t]
    embed = ks.to_numpy_f64(embed_t) * (1.0 / std)      # unit-scale embeddings: livelier attention
    n = int(np.sum(group_len)) + instr_len
    ids = ks.make_token_ids(n, shape.vocab, seed)
    sh = oracle_shape(shape, oracle_storage)
    kb, vb = ko.precompute_group_caches(sh, layers, embed, ids, list(group_len))
    return sh, layers, embed, ids, kb, vb
