"""Parity at the benchmark's full size (Qwen-14B-shaped layer, 33 024-token prompt), in the launch
configuration bench.py times: one selective layer teacher-forced on seeded inputs, checked against
the CPU oracle on the whole refreshed K/V cache, on sampled output rows, and on sampled rows of the
score matrix.  Inputs are seeded draws (keep_synth); nothing the oracle reads comes from the GPU."""
import numpy as np
import pytest
import torch

import keep_synth as ks
from oracle import keep_oracle as ko
from gpu_util import max_rel, to_np

pytestmark = pytest.mark.gpu
TOL = 2e-2


def test_fullsize_selective_layer_sampled():
    from paper_2602_23592_amd import KeepContext, KeepPrompt
    w = ks.workload("qwen14b_32k")
    s = w.shape
    one = ks.ModelShape(1, s.hidden, s.n_q_heads, s.n_kv_heads, s.head_dim, s.ffn_dim, s.vocab, s.rope_theta,
                        s.rms_eps, s.storage)
    glen, kinds = ks.group_lengths(w)
    glist = [int(v) for v in glen]
    G, lq = len(glist), w.instr_len
    n_tokens = w.mem_tokens + lq
    # seeded set that fills the layer-1 token budget of the benchmark schedule
    ratios = ks.ratio_schedule(w.ratio, s.n_layers, w.schedule)
    rng = np.random.Generator(np.random.PCG64(5))
    left, groups = ko.budget_tokens(float(ratios[1]), w.mem_tokens), []
    for g in rng.permutation(G):
        if glist[g] <= left:
            groups.append(int(g))
            left -= glist[g]
    groups.sort()
    m = len(groups)
    # inputs: one layer of weights (with biases), random group caches, random hidden rows
    lw_t = ks.make_layer_weights(one, 0, "cpu", bias=True, norm_jitter=0.1)
    kb_t, vb_t = ks.make_random_group_cache(one, glist, 0, seed=7)
    n_rows = sum(glist[g] for g in groups) + lq
    x_t = ks.make_random_rows(n_rows, s.hidden, s.storage, seed=11)
    ids = ks.make_token_ids(n_tokens, s.vocab, 0)
    embed_t = ks.make_embedding(one, "cpu", rows=8)               # not used (x_in is given); ids clipped below
    # ---- GPU
    dev = "cuda"
    lw_d = {k: (None if v is None else v.to(dev)) for k, v in lw_t.items()}
    ctx = KeepContext(ks.ModelShape(1, s.hidden, s.n_q_heads, s.n_kv_heads, s.head_dim, s.ffn_dim, 8, s.rope_theta,
                                    s.rms_eps, s.storage), [lw_d], embed_t.to(dev), n_tokens, G)
    assert ctx.uses_mfma
    kb_d = [[t.to(dev) for t in kb_t]]
    vb_d = [[t.to(dev) for t in vb_t]]
    pr = KeepPrompt(glist, lq, ids % 8, kb_d, vb_d, 1, group_kind=kinds)
    kc = torch.zeros((n_tokens, s.n_kv_heads, s.head_dim), dtype=torch.bfloat16, device=dev)
    vc = torch.zeros_like(kc)
    x_out = torch.empty((n_rows, s.hidden), dtype=torch.bfloat16, device=dev)
    ctx.recompute_layer(pr, 0, groups, x_t.to(dev), x_out, kc, vc)
    nxt, runs, S = ctx.score_groups(pr, 0, groups, float(ratios[2]), w.hops, 1)
    torch.cuda.synchronize()
    # ---- oracle (float64): K/V refresh of every row; attention/FFN and score rows for sampled blocks
    sh = ko.Shape(1, s.hidden, s.n_q_heads, s.n_kv_heads, s.head_dim, s.ffn_dim, 8, s.rope_theta, s.rms_eps, s.storage)
    lw = {k: (None if v is None else ks.to_numpy_f64(v)) for k, v in lw_t.items()}
    kb = [ks.to_numpy_f64(t) for t in kb_t]
    vb = [ks.to_numpy_f64(t) for t in vb_t]
    kh, vh = ko.realign_concat(sh, kb, vb, glist, lq)
    x_np = ks.to_numpy_f64(x_t)
    small = [i for i, g in enumerate(groups) if glist[g] <= 64]
    blocks = sorted({small[0], small[len(small) // 2], small[-1]})           # three 64-token memories
    xo_ref, lse_ref, S_ref = ko.selective_layer(sh, lw, x_np, groups, glist, lq, kh, vh, score_blocks=blocks + [m])
    # whole cache
    ek, ev = max_rel(to_np(kc), kh), max_rel(to_np(vc), vh)
    # sampled output rows: the rows of the sampled blocks and of the instruction
    starts = np.concatenate([[0], np.cumsum([glist[g] for g in groups])])
    rows = np.concatenate([np.arange(starts[b], starts[b + 1]) for b in blocks] + [np.arange(starts[m], starts[m] + lq)])
    ex = max_rel(to_np(x_out[torch.from_numpy(rows).to(dev)]), xo_ref)
    es = np.nanmax(np.abs(S[blocks + [m]] - S_ref[blocks + [m]])) / np.nanmax(S_ref[blocks + [m]])
    print("full size: rows %d groups %d  K %.2e V %.2e X(sampled %d rows) %.2e S(sampled %d rows) %.2e"
          % (n_rows, m, ek, ev, len(rows), ex, len(blocks) + 1, es))
    assert ek < TOL and ev < TOL and ex < TOL and es < TOL
    # the device's selection is the oracle's selection applied to the device's scores
    want, want_runs = ko.select_multihop(S, groups, glist, float(ratios[2]), w.hops, ko.BUDGET_TOKENS)
    assert nxt == want and runs == want_runs
