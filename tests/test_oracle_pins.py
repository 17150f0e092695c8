"""Pins of the CPU oracle against things other than itself (no GPU).

The paper (KEEP) prints no formula and no numeric worked example that survives,
so every pin is a fixed point of the method, an invariant the text states, a
closed form that the mathematics gives, an independent library expression, or
brute force on tiny inputs.
"""
import itertools
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import keep_synth as ks
from oracle import keep_oracle as ko
from oracle_util import layer_to_numpy, oracle_shape, small_problem, small_shape


# ----------------------------------------------------------------------------
# dense decoder layer: independent PyTorch-CPU expression of the textbook layer
# ----------------------------------------------------------------------------
def _torch_rope_complex(x, positions, theta):
    """RoPE written with complex numbers: the pair (x_j, x_{j+dh/2}) is one complex
    number multiplied by exp(i p theta^(-2j/dh))."""
    n, h, dh = x.shape
    half = dh // 2
    inv = torch.tensor([theta ** (-2.0 * j / dh) for j in range(half)], dtype=torch.float64)
    ang = positions.to(torch.float64)[:, None] * inv[None, :]
    z = torch.complex(x[..., :half], x[..., half:]) * torch.polar(torch.ones_like(ang), ang)[:, None, :]
    return torch.cat([z.real, z.imag], dim=-1)


def _torch_dense_layer(sh, w, x, positions):
    t = {k: (None if v is None else torch.from_numpy(v)) for k, v in w.items()}
    x = torch.from_numpy(x)
    n = x.shape[0]
    h = F.rms_norm(x, (sh.hidden,), t["ln1"], sh.rms_eps)
    q = F.linear(h, t["wq"], t["bq"]).view(n, sh.n_q_heads, sh.head_dim)
    k = F.linear(h, t["wk"], t["bk"]).view(n, sh.n_kv_heads, sh.head_dim)
    v = F.linear(h, t["wv"], t["bv"]).view(n, sh.n_kv_heads, sh.head_dim)
    pos = torch.from_numpy(np.asarray(positions))
    q = _torch_rope_complex(q, pos, sh.rope_theta)
    k = _torch_rope_complex(k, pos, sh.rope_theta)
    o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None], v.transpose(0, 1)[None],
                                       is_causal=True, enable_gqa=True)[0].transpose(0, 1)
    x = x + F.linear(o.reshape(n, -1), t["wo"])
    h2 = F.rms_norm(x, (sh.hidden,), t["ln2"], sh.rms_eps)
    x = x + F.linear(F.silu(F.linear(h2, t["wgate"])) * F.linear(h2, t["wup"]), t["wdown"])
    return x.numpy(), k.numpy(), v.numpy()


@pytest.mark.parametrize("first_pos", [0, 37])
def test_dense_layer_matches_torch_expression(first_pos):
    shape = small_shape(n_q_heads=6, n_kv_heads=2, head_dim=8, hidden=48)
    sh = oracle_shape(shape, "f64")
    w = layer_to_numpy(ks.make_layer_weights(shape, 0, std=0.3, bias=True, norm_jitter=0.2))
    rng = np.random.default_rng(3)
    x = rng.standard_normal((11, shape.hidden))
    pos = np.arange(first_pos, first_pos + 11)
    xo, k, v = ko.dense_layer(sh, w, x, pos)
    xt, kt, vt = _torch_dense_layer(sh, w, x, pos)
    np.testing.assert_allclose(k, kt, rtol=0, atol=1e-12)
    np.testing.assert_allclose(v, vt, rtol=0, atol=1e-12)
    np.testing.assert_allclose(xo, xt, rtol=0, atol=1e-11)


# ----------------------------------------------------------------------------
# RoPE: composition and the relative-position property
# ----------------------------------------------------------------------------
def test_rope_rotations_compose():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 3, 16))
    a = np.array([0, 3, 100, 7, 65535])
    b = np.array([9, 0, 23, 4000, 1])
    lhs = ko.rotate(ko.rotate(x, a, 1e6), b, 1e6)
    rhs = ko.rotate(x, a + b, 1e6)
    np.testing.assert_allclose(lhs, rhs, atol=1e-9)
    np.testing.assert_allclose(ko.rotate(x, np.zeros(5, dtype=int), 1e6), x, atol=0)
    # a rotation keeps the norm of every (j, j+dh/2) pair, and turns pair 0 by exactly p radians
    y = ko.rotate(x, a, 1e6)
    np.testing.assert_allclose(y[..., 0] ** 2 + y[..., 8] ** 2, x[..., 0] ** 2 + x[..., 8] ** 2, rtol=1e-12)
    e = np.zeros((1, 1, 16)); e[0, 0, 0] = 1.0
    r = ko.rotate(e, np.array([2]), 1e6)
    assert abs(r[0, 0, 0] - math.cos(2.0)) < 1e-15 and abs(r[0, 0, 8] - math.sin(2.0)) < 1e-15


def test_group_alone_at_shifted_positions_gives_rotated_keys_same_values():
    """Attention depends on relative positions only: a group prefilled on its own at
    positions off..off+n-1 has the same V and hidden states as at 0..n-1, and its K is
    the local K rotated on by off.  This is what makes re-alignment of cached keys valid."""
    shape = small_shape()
    sh, layers, embed, ids, _, _ = small_problem(shape, [9], 1)
    k0, v0, x0 = ko.dense_prefill(sh, layers, embed, ids[:9], 0)
    k1, v1, x1 = ko.dense_prefill(sh, layers, embed, ids[:9], 41)
    for l in range(shape.n_layers):
        np.testing.assert_allclose(v1[l], v0[l], atol=1e-10)
        np.testing.assert_allclose(k1[l], ko.rotate(k0[l], np.full(9, 41), sh.rope_theta), atol=1e-10)
    np.testing.assert_allclose(x1, x0, atol=1e-10)


# ----------------------------------------------------------------------------
# fixed points of the whole method
# ----------------------------------------------------------------------------
GROUPS = [5, 3, 7, 4]
LQ = 6


def test_full_ratio_equals_dense_causal_prefill():
    """Recomputing every memory at every layer is a dense prefill of the joined prompt."""
    shape = small_shape(n_layers=3)
    sh, layers, embed, ids, kb, vb = small_problem(shape, GROUPS, LQ)
    r = ko.keep_prefill(sh, layers, embed, ids, GROUPS, LQ, kb, vb, [1.0, 1.0, 1.0], 2)
    kd, vd, xd = ko.dense_prefill(sh, layers, embed, ids, 0)
    for l in range(shape.n_layers):
        np.testing.assert_allclose(r["k_hat"][l], kd[l], atol=1e-10)
        np.testing.assert_allclose(r["v_hat"][l], vd[l], atol=1e-10)
        assert r["sets"][l] == [0, 1, 2, 3]
    np.testing.assert_allclose(r["x_final"], xd[-LQ:], atol=1e-10)
    # and it differs from full reuse, so the test can fail
    r0 = ko.keep_prefill(sh, layers, embed, ids, GROUPS, LQ, kb, vb, [0.0, 0.0, 0.0], 1)
    assert np.abs(r0["x_final"] - xd[-LQ:]).max() > 1e-3


def test_zero_ratio_is_rerotated_concatenation():
    """Recomputing nothing leaves the joined cache = cached V, cached K rotated on by the
    group offset; only instruction rows are computed (full KV reuse, Section 3)."""
    shape = small_shape(n_layers=2)
    sh, layers, embed, ids, kb, vb = small_problem(shape, GROUPS, LQ)
    r = ko.keep_prefill(sh, layers, embed, ids, GROUPS, LQ, kb, vb, [0.0, 0.0], 3)
    off = np.concatenate([[0], np.cumsum(GROUPS)])
    for l in range(shape.n_layers):
        assert r["sets"][l] == []
        for g, n in enumerate(GROUPS):
            np.testing.assert_array_equal(r["v_hat"][l][off[g]:off[g] + n], vb[l][g])
            # independent expression of the shift: complex rotation by off_g
            kt = _torch_rope_complex(torch.from_numpy(kb[l][g]), torch.full((n,), int(off[g])), sh.rope_theta)
            np.testing.assert_allclose(r["k_hat"][l][off[g]:off[g] + n], kt.numpy(), atol=1e-12)
    # instruction K/V at layer 0 depend on the embeddings alone: same as in the dense prefill
    kd, vd, _ = ko.dense_prefill(sh, layers, embed, ids, 0)
    np.testing.assert_allclose(r["k_hat"][0][-LQ:], kd[0][-LQ:], atol=1e-10)
    np.testing.assert_allclose(r["v_hat"][0][-LQ:], vd[0][-LQ:], atol=1e-10)
    # x_final: the instruction prefilled over the joined cache, written out by hand for one head layout
    x = embed[ids[-LQ:]]
    for l in range(shape.n_layers):
        x, _, _ = ko.selective_layer(sh, layers[l], x, [], GROUPS, LQ, r["k_hat"][l].copy(), r["v_hat"][l].copy(),
                                     want_scores=False)
    np.testing.assert_allclose(r["x_final"], x, atol=1e-12)


def test_lone_group_reproduces_its_own_cache():
    shape = small_shape(n_layers=3)
    sh, layers, embed, ids, kb, vb = small_problem(shape, [11], 3)
    r = ko.keep_prefill(sh, layers, embed, ids, [11], 3, kb, vb, [1.0, 1.0, 1.0], 2)
    for l in range(shape.n_layers):
        np.testing.assert_allclose(r["k_hat"][l][:11], kb[l][0], atol=1e-10)
        np.testing.assert_allclose(r["v_hat"][l][:11], vb[l][0], atol=1e-10)


def test_first_group_and_layer0_invariances():
    """Nothing precedes the first group, so recomputing it gives back its cache at every
    layer; layer-0 K/V depend on embeddings only, so recomputing any group at layer 0
    gives back its re-rotated cache."""
    shape = small_shape(n_layers=3)
    sh, layers, embed, ids, kb, vb = small_problem(shape, GROUPS, LQ)
    forced = [[0, 1, 2, 3], [0, 2, 3], [0, 3]]
    r = ko.keep_prefill(sh, layers, embed, ids, GROUPS, LQ, kb, vb, [1.0, 0.75, 0.5], 2, forced_sets=forced)
    assert r["sets"] == forced
    reuse = ko.keep_prefill(sh, layers, embed, ids, GROUPS, LQ, kb, vb, [0.0, 0.0, 0.0], 1)
    for l in range(3):
        np.testing.assert_allclose(r["k_hat"][l][:5], kb[l][0], atol=1e-10)
        np.testing.assert_allclose(r["v_hat"][l][:5], vb[l][0], atol=1e-10)
    nm = sum(GROUPS)
    np.testing.assert_allclose(r["k_hat"][0][:nm], reuse["k_hat"][0][:nm], atol=1e-10)
    np.testing.assert_allclose(r["v_hat"][0][:nm], reuse["v_hat"][0][:nm], atol=1e-10)
    # a group that is NOT recomputed keeps its re-rotated cache exactly
    np.testing.assert_array_equal(r["k_hat"][1][5:8], reuse["k_hat"][1][5:8])
    np.testing.assert_array_equal(r["v_hat"][2][8:15], reuse["v_hat"][2][8:15])
    # a later group that IS recomputed at layer >= 1 differs from its cache (cross-attention recovered)
    assert np.abs(r["v_hat"][1][15:19] - reuse["v_hat"][1][15:19]).max() > 1e-4


def test_selective_equals_dense_for_recomputed_prefix():
    """If the recomputed set is a prefix of the groups at every layer, those groups'
    K/V equal the dense prefill's (they see only recomputed, hence exact, predecessors)."""
    shape = small_shape(n_layers=3)
    sh, layers, embed, ids, kb, vb = small_problem(shape, GROUPS, LQ)
    forced = [[0, 1, 2, 3], [0, 1, 2], [0, 1]]
    r = ko.keep_prefill(sh, layers, embed, ids, GROUPS, LQ, kb, vb, [1.0, 0.75, 0.5], 1, forced_sets=forced)
    kd, vd, _ = ko.dense_prefill(sh, layers, embed, ids, 0)
    np.testing.assert_allclose(r["k_hat"][1][:15], kd[1][:15], atol=1e-10)
    np.testing.assert_allclose(r["v_hat"][2][:8], vd[2][:8], atol=1e-10)


def test_only_rows_matches_full_layer():
    shape = small_shape(n_layers=1)
    sh, layers, embed, ids, kb, vb = small_problem(shape, GROUPS, LQ)
    kh, vh = ko.realign_concat(sh, kb[0], vb[0], GROUPS, LQ)
    groups = [1, 3]
    pos = ko.rows_of(groups, GROUPS, LQ)
    x = np.random.default_rng(5).standard_normal((len(pos), shape.hidden))
    k1, v1 = kh.copy(), vh.copy()
    xo, lse, _ = ko.selective_layer(sh, layers[0], x, groups, GROUPS, LQ, k1, v1)
    k2, v2 = kh.copy(), vh.copy()
    pick = np.array([0, 4, len(pos) - 1])
    xs, lse_s, _ = ko.selective_layer(sh, layers[0], x, groups, GROUPS, LQ, k2, v2, want_scores=False, only_rows=pick)
    np.testing.assert_array_equal(k1, k2)
    np.testing.assert_allclose(xs, xo[pick], atol=1e-12)
    np.testing.assert_allclose(lse_s, lse[pick], atol=1e-12)


# ----------------------------------------------------------------------------
# scores
# ----------------------------------------------------------------------------
def _attention_probs_by_hand(sh, w, x, pos, k_hat):
    """P[h, t, j] with explicit loops (tiny sizes only)."""
    q, _, _ = ko.project_qkv(sh, w, x, pos)
    rep = sh.n_q_heads // sh.n_kv_heads
    n_total = k_hat.shape[0]
    p = np.zeros((sh.n_q_heads, len(pos), n_total))
    for h in range(sh.n_q_heads):
        for t in range(len(pos)):
            sc = np.array([q[t, h] @ k_hat[j, h // rep] / math.sqrt(sh.head_dim) for j in range(pos[t] + 1)])
            e = np.exp(sc - sc.max())
            p[h, t, :pos[t] + 1] = e / e.sum()
    return p


def test_scores_match_loop_definition_and_conserve_mass():
    shape = small_shape(n_layers=1)
    sh, layers, embed, ids, kb, vb = small_problem(shape, GROUPS, LQ)
    kh, vh = ko.realign_concat(sh, kb[0], vb[0], GROUPS, LQ)
    groups = [0, 2, 3]
    pos = ko.rows_of(groups, GROUPS, LQ)
    x = np.random.default_rng(1).standard_normal((len(pos), shape.hidden))
    _, lse, S = ko.selective_layer(sh, layers[0], x, groups, GROUPS, LQ, kh, vh)
    p = _attention_probs_by_hand(sh, layers[0], x, pos, kh)       # kh now holds refreshed K
    np.testing.assert_allclose(p.sum(axis=2), 1.0, atol=1e-12)
    off = np.concatenate([[0], np.cumsum(GROUPS)])
    row_blocks = {}
    c = 0
    for g in groups:
        row_blocks[g] = range(c, c + GROUPS[g]); c += GROUPS[g]
    row_blocks["q"] = range(c, c + LQ)
    for i, a in enumerate(groups + ["q"]):
        for j, b in enumerate(groups):
            want = 0.0
            if a != b:
                for h in range(sh.n_q_heads):
                    for t in row_blocks[a]:
                        for s_ in range(off[b], off[b + 1]):
                            want += p[h, t, s_]
                want /= sh.n_q_heads * len(row_blocks[a]) * GROUPS[b]
            assert abs(S[i, j] - want) < 1e-13
    # causality: a memory sends nothing to memories placed after it
    for i, a in enumerate(groups):
        for j, b in enumerate(groups):
            if b >= a:
                assert S[i, j] == 0.0
    assert (S[-1] > 0).all()
    # log-sum-exp really is the log of the softmax denominator
    q, _, _ = ko.project_qkv(sh, layers[0], x, pos)
    t, h = 3, 1
    sc = np.array([q[t, h] @ kh[j, h // 2] / math.sqrt(sh.head_dim) for j in range(pos[t] + 1)])
    assert abs(lse[t, h] - math.log(np.exp(sc).sum())) < 1e-12


def test_uniform_attention_gives_harmonic_closed_form():
    """With Wq = 0 (and no q bias) every visible key gets probability 1/(p_t+1), so
    S[a, b] = (1/len_a) * sum_{t in a} 1/(p_t+1) for b before a: differences of
    harmonic numbers, whatever the other weights are."""
    shape = small_shape(n_layers=1)
    sh, layers, embed, ids, kb, vb = small_problem(shape, GROUPS, LQ, bias=False)
    w = dict(layers[0]); w["wq"] = np.zeros_like(w["wq"])
    kh, vh = ko.realign_concat(sh, kb[0], vb[0], GROUPS, LQ)
    groups = [0, 1, 2, 3]
    pos = ko.rows_of(groups, GROUPS, LQ)
    x = np.random.default_rng(2).standard_normal((len(pos), shape.hidden))
    _, _, S = ko.selective_layer(sh, w, x, groups, GROUPS, LQ, kh, vh)
    off = np.concatenate([[0], np.cumsum(GROUPS), [sum(GROUPS) + LQ]])
    harm = lambda n: sum(1.0 / i for i in range(1, n + 1))
    for i in range(5):
        mean_inv = (harm(off[i + 1]) - harm(off[i])) / (off[i + 1] - off[i])
        for j in range(4):
            want = mean_inv if j < i else 0.0
            assert abs(S[i, j] - want) < 1e-14


# ----------------------------------------------------------------------------
# selection
# ----------------------------------------------------------------------------
def test_budget_rounding():
    assert ko.budget_count(0.15, 64, 64) == 10          # ceil(9.6)
    assert ko.budget_count(0.125, 64, 64) == 8          # exact product stays
    assert ko.budget_count(0.1, 10, 10) == 1            # binary32(0.1)*10 is a hair above 1
    assert ko.budget_count(0.1, 272, 272) == 28
    assert ko.budget_count(0.5, 8, 3) == 3              # never more than the candidates
    assert ko.budget_count(0.0, 8, 8) == 0
    assert ko.budget_tokens(0.1, 1000) == 100
    assert ko.budget_tokens(0.15, 1024) == 153


def _brute_topk(imp, k):
    """Best k-subset by enumeration: maximise the sorted importance vector
    lexicographically, then minimise the indices."""
    best = None
    for sub in itertools.combinations(range(len(imp)), k):
        key = (tuple(sorted((-float(imp[b]) for b in sub))), sub)
        if best is None or key < best[0]:
            best = (key, sub)
    return list(best[1]) if best else []


def test_single_hop_is_topk_of_query_row_bruteforce():
    rng = np.random.default_rng(4)
    for trial in range(30):
        m = int(rng.integers(2, 8))
        S = rng.random((m + 1, m)).astype(np.float32)
        if trial % 3 == 0:                      # force ties
            S[m] = np.round(S[m] * 3) / 3
        glen = [1] * m
        for k in range(1, m):
            ratio = k / m
            got, runs = ko.select_multihop(S, list(range(m)), glen, ratio, 1)
            assert runs == 1
            assert got == _brute_topk(S[m] / S[m].sum(dtype=np.float32), k)


def test_token_budget_walk_bruteforce():
    """Token mode walks the importance order and takes a memory iff it still fits."""
    rng = np.random.default_rng(6)
    for trial in range(20):
        m = int(rng.integers(2, 7))
        S = np.zeros((m + 1, m), dtype=np.float32)
        S[m] = rng.permutation(m) + 1          # distinct importances
        glen = [int(v) for v in rng.integers(1, 9, size=m)]
        total = sum(glen)
        budget_tok = int(rng.integers(1, total))
        ratio = (budget_tok + 0.5) / total
        got, _ = ko.select_multihop(S, list(range(m)), glen, ratio, 1, ko.BUDGET_TOKENS)
        order = sorted(range(m), key=lambda b: -S[m, b])
        used, want = 0, []
        for b in order:
            if used + glen[b] <= budget_tok:
                want.append(b); used += glen[b]
        assert got == sorted(want)
        assert sum(glen[b] for b in got) <= budget_tok


def test_tie_rule_lower_index_wins():
    S = np.zeros((5, 4), dtype=np.float32)
    S[4] = [0.25, 0.25, 0.25, 0.25]
    got, _ = ko.select_multihop(S, [3, 5, 8, 9], [1] * 10, 0.2, 1)
    assert got == [3, 5]


def test_no_memory_to_memory_attention_is_stable_at_second_hop():
    S = np.zeros((6, 5), dtype=np.float32)
    S[5] = [0.1, 0.5, 0.05, 0.3, 0.05]
    got, runs = ko.select_multihop(S, list(range(5)), [1] * 5, 0.4, 4)
    assert got == [1, 3] and runs == 2


def _chain_scores():
    """Five memories; the query attends to memory 4 ("locked door"), which attends to 2
    ("key"), which attends to 0 ("table"): the reasoning chain of Fig. 6 with numbers of
    this repository's own (the figure's numbers are not in the text).  Causal: a memory
    attends only to earlier ones."""
    S = np.zeros((6, 5), dtype=np.float32)
    S[5] = [0.05, 0.10, 0.15, 0.12, 0.58]       # query: door first
    S[4] = [0.02, 0.03, 0.90, 0.05, 0.00]       # door -> key
    S[2] = [0.95, 0.05, 0.00, 0.00, 0.00]       # key -> table
    S[3] = [0.30, 0.30, 0.40, 0.00, 0.00]
    S[1] = [1.00, 0.00, 0.00, 0.00, 0.00]
    return S


def test_multihop_chain_finds_the_table():
    S = _chain_scores()
    glen = [1] * 5
    one, r1 = ko.select_multihop(S, list(range(5)), glen, 0.6, 1)
    assert one == [2, 3, 4] and r1 == 1                   # init only: door, key, memory 3; no table
    # hop 2: importance = (query + rows 2,3,4)/4 -> the table (memory 0) overtakes memory 3
    two, r2 = ko.select_multihop(S, list(range(5)), glen, 0.6, 2)
    assert two == [0, 2, 4] and r2 == 2
    # by hand in float64: I'[0] = (0.05+0.95+0.30+0.02)/4 = 0.33, I'[2] = (0.15+0+0.4+0.9)/4,
    # I'[4] = 0.58/4, I'[3] = (0.12+0.05)/4, I'[1] = (0.10+0.05+0.30+0.03)/4 = 0.12
    many, r4 = ko.select_multihop(S, list(range(5)), glen, 0.6, 8)
    assert r4 <= 8 and set(many) >= {0, 2}
    # the golden file holds the same chain with its expected sets
    import json, os
    gold = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "chain_fig6_style.json")))
    Sg = np.array(gold["scores"], dtype=np.float32)
    for case in gold["cases"]:
        got, runs = ko.select_multihop(Sg, list(range(5)), glen, case["ratio"], case["hops"])
        assert got == case["expect"], case
        assert runs == case["runs"], case


def test_literal_variant_can_drop_first_hop_memories():
    """Averaging over the relevant memories alone (query dropped) removes any memory
    that only the query attends to -- here the first-hop memory 4 -- which is why the
    oracle keeps the query as a source."""
    S = np.zeros((6, 5), dtype=np.float32)
    S[5] = [0.0, 0.0, 0.35, 0.05, 0.60]
    S[4] = [0.05, 0.05, 0.90, 0.0, 0.0]
    S[2] = [0.5, 0.5, 0.0, 0.0, 0.0]
    literal, _ = ko.select_multihop(S, list(range(5)), [1] * 5, 0.4, 2, drop_query=True)
    adopted, _ = ko.select_multihop(S, list(range(5)), [1] * 5, 0.4, 2, drop_query=False)
    assert literal == [0, 2]          # (row2 + row4)/2 = [.275, .275, .45, 0, 0]
    assert adopted == [2, 4]          # (q + row2 + row4)/3 = [.55, .55, 1.25, .05, .6]/3


def test_sets_are_nested_and_sized_by_budget():
    shape = small_shape(n_layers=4)
    groups = [4, 6, 3, 5, 4, 7, 2, 5]
    sh, layers, embed, ids, kb, vb = small_problem(shape, groups, 5)
    ratios = [1.0, 0.75, 0.5, 0.25]
    r = ko.keep_prefill(sh, layers, embed, ids, groups, 5, kb, vb, ratios, 3)
    assert r["sets"][0] == list(range(8))
    for l in range(1, 4):
        assert set(r["sets"][l]) <= set(r["sets"][l - 1])
        assert len(r["sets"][l]) == min(len(r["sets"][l - 1]), math.ceil(ratios[l] * 8 - 1e-3))
        assert r["sets"][l] == sorted(r["sets"][l])
    # token mode: budget respected
    rt = ko.keep_prefill(sh, layers, embed, ids, groups, 5, kb, vb, ratios, 3, ko.BUDGET_TOKENS)
    for l in range(1, 4):
        assert set(rt["sets"][l]) <= set(rt["sets"][l - 1])
        assert sum(groups[g] for g in rt["sets"][l]) <= math.floor(ratios[l] * sum(groups) + 1e-3)


def test_float32_and_float64_oracle_agree():
    shape = small_shape(n_layers=2)
    sh, layers, embed, ids, kb, vb = small_problem(shape, GROUPS, LQ)
    forced = [[0, 1, 2, 3], [1, 3]]
    a = ko.keep_prefill(sh, layers, embed, ids, GROUPS, LQ, kb, vb, [1.0, 0.5], 2, forced_sets=forced)
    l32 = [{k: (None if v is None else v.astype(np.float32)) for k, v in w.items()} for w in layers]
    kb32 = [[b.astype(np.float32) for b in row] for row in kb]
    vb32 = [[b.astype(np.float32) for b in row] for row in vb]
    b = ko.keep_prefill(sh, l32, embed.astype(np.float32), ids, GROUPS, LQ, kb32, vb32, [1.0, 0.5], 2,
                        forced_sets=forced, dtype=np.float32)
    assert b["x_final"].dtype == np.float32
    np.testing.assert_allclose(b["x_final"], a["x_final"], atol=2e-4, rtol=1e-4)
    np.testing.assert_allclose(b["scores"][0], a["scores"][0], atol=1e-6)


def test_bf16_storage_rounds_only_the_cache():
    shape = small_shape(n_layers=1)
    sh, layers, embed, ids, kb, vb = small_problem(shape, GROUPS, LQ, oracle_storage="bf16")
    kh, vh = ko.realign_concat(sh, kb[0], vb[0], GROUPS, LQ)
    bits = ks.bf16_bits_from_f32(kh.astype(np.float32))
    np.testing.assert_array_equal(ks.f32_from_bf16_bits(bits).astype(np.float64), kh)   # already bf16 values
    assert ko.round_to_storage(np.array([1.00390625]), "bf16")[0] == 1.0                # tie to even
    assert ko.round_to_storage(np.array([1.01171875]), "bf16")[0] == 1.015625           # tie to even (up)


def test_score_blocks_matches_full_scores():
    shape = small_shape(n_layers=1)
    sh, layers, embed, ids, kb, vb = small_problem(shape, GROUPS, LQ)
    kh, vh = ko.realign_concat(sh, kb[0], vb[0], GROUPS, LQ)
    groups = [0, 1, 3]
    pos = ko.rows_of(groups, GROUPS, LQ)
    x = np.random.default_rng(5).standard_normal((len(pos), shape.hidden))
    xo, lse, S = ko.selective_layer(sh, layers[0], x, groups, GROUPS, LQ, kh.copy(), vh.copy())
    xs, lse_s, Ss = ko.selective_layer(sh, layers[0], x, groups, GROUPS, LQ, kh.copy(), vh.copy(), score_blocks=[3, 1])
    np.testing.assert_allclose(Ss[[1, 3]], S[[1, 3]], atol=1e-15)
    assert np.isnan(Ss[[0, 2]]).all()
    rows = np.concatenate([np.arange(5, 8), np.arange(12, 12 + LQ)])     # block 1 = group 1 (3 rows), block 3 = query
    np.testing.assert_allclose(xs, xo[rows], atol=1e-12)
