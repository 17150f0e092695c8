"""Parity at the full size of every benchmark workload (the Qwen-14B-shaped 33 024-token prompt that bench.py
times by default, and the 7B / 32B / 64k-token shapes), in the launch configuration bench.py uses: one
selective layer teacher-forced on seeded inputs, checked against
the CPU oracle on the whole refreshed K/V cache, on sampled output rows, and on sampled rows of the
score matrix.  Inputs are seeded draws (keep_synth); nothing the oracle reads comes from the GPU."""
import numpy as np
import pytest
import torch

import keep_synth as ks
from oracle import keep_oracle as ko
from gpu_util import max_rel, mean_rel, to_np, update_err, layer_state_err

pytestmark = pytest.mark.gpu
TOL = 2e-2


@pytest.mark.parametrize("workload", ["qwen14b_32k", "qwen7b_16k", "qwen32b_32k_host", "qwen14b_64k_stress"])
def test_fullsize_selective_layer_sampled(workload):
    from paper_2602_23592_amd import KeepContext, KeepPrompt
    from paper_2602_23592_amd.binding import KEEP_BUDGET_TOKENS, KEEP_BUDGET_GROUP_COUNT
    w = ks.workload(workload)
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
    tokens_mode = w.budget == "tokens"
    if tokens_mode:
        left, groups = ko.budget_tokens(float(ratios[1]), w.mem_tokens), []
        for g in rng.permutation(G):
            if glist[g] <= left:
                groups.append(int(g))
                left -= glist[g]
        groups.sort()
    else:
        groups = sorted(int(g) for g in rng.choice(G, size=ko.budget_count(float(ratios[1]), G, G), replace=False))
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
    from paper_2602_23592_amd.binding import KEEP_STATE_ATTN_OUT, KEEP_STATE_LSE
    o_dev = ctx.read_layer_state(KEEP_STATE_ATTN_OUT, n_rows)
    lse_dev = ctx.read_layer_state(KEEP_STATE_LSE, n_rows)
    mode = KEEP_BUDGET_TOKENS if tokens_mode else KEEP_BUDGET_GROUP_COUNT
    nxt, runs, S = ctx.score_groups(pr, 0, groups, float(ratios[2]), w.hops, mode)
    torch.cuda.synchronize()
    # ---- oracle (float64): K/V refresh of every row; attention/FFN and score rows for sampled blocks
    sh = ko.Shape(1, s.hidden, s.n_q_heads, s.n_kv_heads, s.head_dim, s.ffn_dim, 8, s.rope_theta, s.rms_eps, s.storage)
    lw = {k: (None if v is None else ks.to_numpy_f64(v)) for k, v in lw_t.items()}
    kb = [ks.to_numpy_f64(t) for t in kb_t]
    vb = [ks.to_numpy_f64(t) for t in vb_t]
    kh, vh = ko.realign_concat(sh, kb, vb, glist, lq)
    x_np = ks.to_numpy_f64(x_t)
    # three of the shorter memories (first, middle, last of those no longer than the median) as score samples
    med = int(np.median([glist[g] for g in groups]))
    small = [i for i, g in enumerate(groups) if glist[g] <= med]
    blocks = sorted({small[0], small[len(small) // 2], small[-1]})
    probe = {}
    xo_ref, lse_ref, S_ref = ko.selective_layer(sh, lw, x_np, groups, glist, lq, kh, vh, score_blocks=blocks + [m],
                                                probe=probe)
    # whole cache
    ek, ev = max_rel(to_np(kc), kh), max_rel(to_np(vc), vh)
    # sampled output rows: the rows of the sampled blocks and of the instruction
    starts = np.concatenate([[0], np.cumsum([glist[g] for g in groups])])
    rows = np.concatenate([np.arange(starts[b], starts[b + 1]) for b in blocks] + [np.arange(starts[m], starts[m] + lq)])
    xo_dev = to_np(x_out[torch.from_numpy(rows).to(dev)])
    ex = max_rel(xo_dev, xo_ref)
    es = np.nanmax(np.abs(S[blocks + [m]] - S_ref[blocks + [m]])) / np.nanmax(S_ref[blocks + [m]])
    # on their own scale: the attention output and log-sum-exp of the sampled rows, and the layer's update
    # (output minus input) of those rows, where the residual stream does not hide an attention error
    eo = max_rel(o_dev[rows].astype(np.float64), probe["attn_out"])
    el = max_rel(lse_dev[rows].astype(np.float64), lse_ref)
    ed, allow = update_err(xo_dev, x_np[rows], xo_ref, "bf16")
    print("full size %s: rows %d groups %d  K %.2e V %.2e X(sampled %d rows) %.2e S(sampled %d rows) %.2e  "
          "attention %.2e lse %.2e update %.2e (format %.1e)"
          % (workload, n_rows, m, ek, ev, len(rows), ex, len(blocks) + 1, es, eo, el, ed, allow))
    assert ek < TOL and ev < TOL and ex < TOL and es < TOL
    assert eo < TOL and el < TOL and ed < TOL + allow
    # the device's selection is the oracle's selection applied to the device's scores
    want, want_runs = ko.select_multihop(S, groups, glist, float(ratios[2]), w.hops,
                                         ko.BUDGET_TOKENS if tokens_mode else ko.BUDGET_GROUP_COUNT)
    assert nxt == want and runs == want_runs


def test_decode_attention_over_the_full_cache_matches_oracle():
    """One new token over the 33 024-row cache of the bench workload's shape (one layer, random cache):
    the launch configuration the decode benchmark times.  The oracle computes the single row directly."""
    import keep_synth as ks
    from oracle import keep_oracle as ko
    from oracle_util import layer_to_numpy, oracle_shape
    from paper_2602_23592_amd import KeepContext
    full = ks.workload("qwen14b_32k").shape
    shape = ks.ModelShape(1, full.hidden, full.n_q_heads, full.n_kv_heads, full.head_dim, full.ffn_dim, 4099,
                          full.rope_theta, full.rms_eps, "bf16")
    n_ctx = 33024
    w_t = ks.make_layer_weights(shape, 0, "cpu")
    embed_t = ks.make_embedding(shape, "cpu")
    g = torch.Generator().manual_seed(5)
    kc = torch.randn((1, n_ctx + 2, shape.n_kv_heads, shape.head_dim), generator=g).to(torch.bfloat16)
    vc = torch.randn((1, n_ctx + 2, shape.n_kv_heads, shape.head_dim), generator=g).to(torch.bfloat16)
    fn = torch.ones(shape.hidden, dtype=torch.bfloat16)
    lm = (0.02 * torch.randn((shape.vocab, shape.hidden), generator=g)).to(torch.bfloat16)
    x_last = (0.5 * torch.randn(shape.hidden, generator=g)).to(torch.bfloat16)
    ctx = KeepContext(shape, [{k: (None if v is None else v.cuda()) for k, v in w_t.items()}], embed_t.cuda(),
                      n_ctx + 2, 1, 0)
    assert ctx.uses_mfma
    kd, vd = kc.cuda(), vc.cuda()
    logits = torch.empty((2, shape.vocab), dtype=torch.float32, device="cuda")
    toks = ctx.decode(fn.cuda(), lm.cuda(), x_last.cuda(), kd, vd, n_ctx, 2, logits_out=logits)
    torch.cuda.synchronize()
    sh = oracle_shape(shape)
    kr, vr = [ks.to_numpy_f64(kc[0])], [ks.to_numpy_f64(vc[0])]
    _, rlg = ko.greedy_decode(sh, [layer_to_numpy(w_t)], ks.to_numpy_f64(embed_t), ks.to_numpy_f64(fn),
                              ks.to_numpy_f64(lm), ks.to_numpy_f64(x_last), kr, vr, n_ctx, 2, forced_tokens=toks)
    lg = logits.cpu().double().numpy()
    for t in range(2):
        e = np.abs(lg[t] - rlg[t]).max() / np.abs(rlg[t]).max()
        print("full-size decode step", t, "logits err %.2e" % e)
        assert e < 2e-2
    assert np.abs(kd[0, n_ctx].cpu().double().numpy() - kr[0][n_ctx]).max() / np.abs(kr[0][n_ctx]).max() < 2e-2
    assert np.abs(vd[0, n_ctx].cpu().double().numpy() - vr[0][n_ctx]).max() / np.abs(vr[0][n_ctx]).max() < 2e-2


def test_fullsize_prefill_layer0_selection_equals_full_matrix_selection():
    """The bench workload's layer 0 -> 1 decision at full size (272 candidates, 33 024 rows, token budget,
    3 hops), where keep_prefill forms the score rows hop by hop: the set must be the one the selector gives
    on the complete score matrix of the same layer (keep_recompute_layer + keep_score_groups), which in turn
    must be the oracle's selection applied to that matrix."""
    from paper_2602_23592_amd import KeepContext, KeepPrompt
    from paper_2602_23592_amd.binding import KEEP_BUDGET_TOKENS
    w = ks.workload("qwen14b_32k")
    s = w.shape
    two = ks.ModelShape(2, s.hidden, s.n_q_heads, s.n_kv_heads, s.head_dim, s.ffn_dim, 4099, s.rope_theta,
                        s.rms_eps, s.storage)
    glen, kinds = ks.group_lengths(w)
    glist = [int(v) for v in glen]
    G, lq = len(glist), w.instr_len
    n_tokens = w.mem_tokens + lq
    dev = "cuda"
    layers = [ks.make_layer_weights(two, l, dev) for l in range(2)]
    embed = ks.make_embedding(two, dev)
    ids = ks.make_token_ids(n_tokens, two.vocab, 0)
    ctx = KeepContext(two, layers, embed, n_tokens, G)
    assert ctx.uses_mfma
    kb = torch.empty((2, w.mem_tokens, s.n_kv_heads, s.head_dim), dtype=torch.bfloat16, device=dev)
    vb = torch.empty_like(kb)
    ctx.precompute_groups(glist, ids[:w.mem_tokens], kb, vb)          # group caches by the library's own dense path
    off = np.concatenate([[0], np.cumsum(glist)]).astype(np.int64)
    k_blocks = [[kb[l, off[g]:off[g + 1]] for g in range(G)] for l in range(2)]
    v_blocks = [[vb[l, off[g]:off[g + 1]] for g in range(G)] for l in range(2)]
    pr = KeepPrompt(glist, lq, ids, k_blocks, v_blocks, 2, group_kind=kinds)
    ratio1 = float(ks.ratio_schedule(w.ratio, s.n_layers, w.schedule)[1])
    kc = torch.empty((2, n_tokens, s.n_kv_heads, s.head_dim), dtype=torch.bfloat16, device=dev)
    vc = torch.empty_like(kc)
    xf = torch.empty((lq, s.hidden), dtype=torch.bfloat16, device=dev)
    sets, rep = ctx.prefill(pr, [1.0, ratio1], w.hops, kc, vc, xf, KEEP_BUDGET_TOKENS, want_report=True)
    x_out = torch.empty((n_tokens, s.hidden), dtype=torch.bfloat16, device=dev)
    ctx.recompute_layer(pr, 0, list(range(G)), None, x_out, kc[0], vc[0])
    nxt, runs, S = ctx.score_groups(pr, 0, list(range(G)), ratio1, w.hops, KEEP_BUDGET_TOKENS)
    torch.cuda.synchronize()
    print("full size layer 0 -> 1: set", sets[1], "hops run", rep.hops_run[0], "| full matrix:", nxt, runs)
    assert sets[1] == nxt and rep.hops_run[0] == runs
    want, want_runs = ko.select_multihop(S, list(range(G)), glist, ratio1, w.hops, ko.BUDGET_TOKENS)
    assert nxt == want and runs == want_runs
    assert rep.ffn_rows[0] == sum(glist[g] for g in nxt) + lq       # evaluation went first: FFN on the survivors only


# ---------------------------------------------------------------------------------------------------------
# The first two layers of the benchmark workload through keep_prefill, as bench.py launches it
# ---------------------------------------------------------------------------------------------------------
_TWO_LAYER_RUN = {}


def _two_layer_run():
    """Layers 0 and 1 of qwen14b_32k through keep_prefill in bench.py's configuration: three streams, token
    budget, 3 hops, 272 candidates (scores hop by hop, attention on demand, evaluation before the FFN, FFN on
    the survivors).  Weights and token ids are the seeded draws of the benchmark; the group caches are seeded
    random blocks (the oracle must not read anything the device produced).  Run once per process."""
    if _TWO_LAYER_RUN:
        return _TWO_LAYER_RUN
    from paper_2602_23592_amd import KeepContext, KeepPrompt
    from paper_2602_23592_amd.binding import KEEP_BUDGET_TOKENS
    w = ks.workload("qwen14b_32k")
    s = w.shape
    two = ks.ModelShape(2, s.hidden, s.n_q_heads, s.n_kv_heads, s.head_dim, s.ffn_dim, 4099, s.rope_theta,
                        s.rms_eps, s.storage)
    glen, kinds = ks.group_lengths(w)
    glist = [int(v) for v in glen]
    G, lq = len(glist), w.instr_len
    n_tokens = w.mem_tokens + lq
    dev = "cuda"
    layers_t = [ks.make_layer_weights(two, l, "cpu") for l in range(2)]
    embed_t = ks.make_embedding(two, "cpu")
    ids = ks.make_token_ids(n_tokens, two.vocab, 0)
    caches = [ks.make_random_group_cache(two, glist, l, seed=7) for l in range(2)]
    streams = [torch.cuda.Stream() for _ in range(3)]
    ctx = KeepContext(two, [{k: (None if v is None else v.to(dev)) for k, v in lw.items()} for lw in layers_t],
                      embed_t.to(dev), n_tokens, G, 0, *streams)
    assert ctx.uses_mfma
    kb_d = [[t.to(dev) for t in caches[l][0]] for l in range(2)]
    vb_d = [[t.to(dev) for t in caches[l][1]] for l in range(2)]
    pr = KeepPrompt(glist, lq, ids, kb_d, vb_d, 2, group_kind=kinds)
    ratio1 = float(ks.ratio_schedule(w.ratio, s.n_layers, w.schedule)[1])
    kc = torch.full((2, n_tokens, s.n_kv_heads, s.head_dim), float("nan"), dtype=torch.bfloat16, device=dev)
    vc = kc.clone()
    xf = torch.empty((lq, s.hidden), dtype=torch.bfloat16, device=dev)
    torch.cuda.synchronize()
    sets, rep = ctx.prefill(pr, [1.0, ratio1], w.hops, kc, vc, xf, KEEP_BUDGET_TOKENS, want_report=True)
    torch.cuda.synchronize()
    # the configuration under test really ran
    assert rep.attn_rows[0] < rep.rows[0] == n_tokens and rep.ffn_rows[0] == rep.rows[1] < n_tokens // 2
    _TWO_LAYER_RUN.update(dict(w=w, two=two, glist=glist, lq=lq, n_tokens=n_tokens, layers_t=layers_t, embed_t=embed_t,
                               ids=ids, caches=caches, ratio1=ratio1, sets=sets, hops_run=rep.hops_run[0],
                               kc=kc.cpu(), vc=vc.cpu(), xf=xf.cpu()))
    ctx.close()
    return _TWO_LAYER_RUN


def _oracle_inputs(r, dtype):
    two = r["two"]
    sh = ko.Shape(2, two.hidden, two.n_q_heads, two.n_kv_heads, two.head_dim, two.ffn_dim, two.vocab, two.rope_theta,
                  two.rms_eps, two.storage)
    lws = [{k: (None if v is None else v.to(torch.float64 if dtype == np.float64 else torch.float32).numpy())
            for k, v in lw.items()} for lw in r["layers_t"]]
    embed = r["embed_t"].to(torch.float64).numpy().astype(dtype)
    return sh, lws, embed


def test_fullsize_first_two_layers_against_the_oracle():
    """What the benchmark's layer 0 leaves behind, against the oracle teacher-forced to the device's sets: the
    whole K/V cache of layer 0 (every row refreshed), the whole K/V cache of layer 1 (survivors refreshed from
    layer 0's output rows, the rest re-aligned) and the final instruction rows.  An error in the hop-by-hop
    attention, the survivor gather or the survivors-only FFN would show in layer 1."""
    r = _two_layer_run()
    glist, lq, sets = r["glist"], r["lq"], r["sets"]
    G = len(glist)
    assert sets[0] == list(range(G)) and 0 < len(sets[1]) < G
    sh, lws, embed = _oracle_inputs(r, np.float64)
    off = ko.group_offsets(glist)
    # layer 0: K/V of all rows; attention, projection and FFN only for the rows that survive
    kb0 = [ks.to_numpy_f64(t) for t in r["caches"][0][0]]
    vb0 = [ks.to_numpy_f64(t) for t in r["caches"][0][1]]
    kh0, vh0 = ko.realign_concat(sh, kb0, vb0, glist, lq)
    x0 = embed[np.asarray(r["ids"])]
    keep_rows = ko.rows_of(sets[1], glist, lq)              # at layer 0 the compact row index is the position
    x1, _, _ = ko.selective_layer(sh, lws[0], x0, sets[0], glist, lq, kh0, vh0, want_scores=False, only_rows=keep_rows)
    ek0, ev0 = max_rel(to_np(r["kc"][0]), kh0), max_rel(to_np(r["vc"][0]), vh0)
    # layer 1: survivors refreshed over the joined cache; only the instruction rows are needed afterwards
    kb1 = [ks.to_numpy_f64(t) for t in r["caches"][1][0]]
    vb1 = [ks.to_numpy_f64(t) for t in r["caches"][1][1]]
    kh1, vh1 = ko.realign_concat(sh, kb1, vb1, glist, lq)
    n1 = len(keep_rows)
    xf_ref, _, _ = ko.selective_layer(sh, lws[1], x1, sets[1], glist, lq, kh1, vh1, want_scores=False,
                                      only_rows=np.arange(n1 - lq, n1))
    ek1, ev1 = max_rel(to_np(r["kc"][1]), kh1), max_rel(to_np(r["vc"][1]), vh1)
    # refreshed rows of layer 1 on their own scale (the re-aligned random blocks dominate the whole-cache norm)
    ek1r = max_rel(to_np(r["kc"][1])[keep_rows], kh1[keep_rows])
    ev1r = max_rel(to_np(r["vc"][1])[keep_rows], vh1[keep_rows])
    ex = max_rel(to_np(r["xf"]), xf_ref)
    ed, allow = update_err(to_np(r["xf"]), x1[n1 - lq:], xf_ref, "bf16")
    print("two layers at full size: set sizes %s  layer 0 K %.2e V %.2e | layer 1 K %.2e V %.2e, refreshed rows K %.2e "
          "V %.2e | x_final %.2e, its layer-1 update %.2e (format %.1e)"
          % ([len(x) for x in sets], ek0, ev0, ek1, ev1, ek1r, ev1r, ex, ed, allow))
    print("  mean relative errors: layer 0 K %.2e V %.2e | layer 1 refreshed rows K %.2e V %.2e | x_final %.2e"
          % (mean_rel(to_np(r["kc"][0]), kh0), mean_rel(to_np(r["vc"][0]), vh0),
             mean_rel(to_np(r["kc"][1])[keep_rows], kh1[keep_rows]), mean_rel(to_np(r["vc"][1])[keep_rows], vh1[keep_rows]),
             mean_rel(to_np(r["xf"]), xf_ref)))
    assert not torch.isnan(r["kc"]).any() and not torch.isnan(r["vc"]).any()
    assert max(ek0, ev0, ek1, ev1, ek1r, ev1r, ex) < TOL and ed < TOL + allow


def test_fullsize_layer0_selection_overlap_with_the_free_running_oracle():
    """The device's bf16 decision for layer 1 (272 candidates, token budget, 3 hops) against the oracle deciding
    on its own scores: the oracle forms the rows of S that its own propagation reads (the query's, then those of
    each selection's memories), nothing is taken from the device.  Reports the share of the oracle's recomputed
    tokens that the device recomputes too, and asserts the benchmark spec's bound."""
    r = _two_layer_run()
    glist, lq, w = r["glist"], r["lq"], r["w"]
    G = len(glist)
    sh, lws, embed = _oracle_inputs(r, np.float32)            # binary32 oracle: the selection arithmetic is binary32
    kb0 = [t.float().numpy() for t in r["caches"][0][0]]
    vb0 = [t.float().numpy() for t in r["caches"][0][1]]
    x0 = embed[np.asarray(r["ids"])]
    groups = list(range(G))
    S = np.zeros((G + 1, G), dtype=np.float32)
    known = set()

    def fill(blocks):
        kh0, vh0 = ko.realign_concat(sh, kb0, vb0, glist, lq, dtype=np.float32)
        _, _, Sb = ko.selective_layer(sh, lws[0], x0, groups, glist, lq, kh0, vh0, score_blocks=sorted(blocks))
        for b in blocks:
            S[b] = Sb[b]
            known.add(b)

    fill([G])                                                  # the query's row
    sel, runs = None, 0
    for h in range(1, w.hops + 1):
        sel, runs = ko.select_multihop(S, groups, glist, r["ratio1"], h, ko.BUDGET_TOKENS)
        if runs < h:
            break                                              # converged before the hop limit
        missing = [b for b in sel if b not in known]
        if h < w.hops and missing:
            fill(missing)                                      # the next selection reads these rows
    tok = lambda gs: sum(glist[g] for g in gs)
    dev = r["sets"][1]
    share = tok(set(dev) & set(sel)) / max(1, tok(sel))
    print("layer 0 -> 1 at full size: device set %s (%d tokens, %d selections) | free-running oracle %s (%d tokens, "
          "%d selections) | token overlap %.4f" % (dev, tok(dev), r["hops_run"], sel, tok(sel), runs, share))
    assert share >= 0.99
