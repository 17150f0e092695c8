"""Pins of the oracle's token-granularity variant (Section 3; Section 4.2, "System advantage") against things
other than itself: dense prefill, the already pinned memory-granularity path, invariances of independently
cached blocks, closed forms and brute force.  No GPU."""
import itertools

import numpy as np
import pytest

import keep_synth as ks
from oracle import keep_oracle as ko
from oracle_util import oracle_shape, small_problem, small_shape

GROUPS, LQ = [5, 9, 3, 7], 4


def _problem(seed=0, n_layers=3):
    shape = small_shape(n_layers=n_layers)
    return shape, small_problem(shape, GROUPS, LQ, seed=seed)


def test_ratio_one_is_dense_prefill_and_ratio_zero_is_pure_reuse():
    shape, (sh, layers, embed, ids, kb, vb) = _problem()
    kd, vd, xd = ko.dense_prefill(sh, layers, embed, ids, 0)
    r = ko.keep_prefill_tokens(sh, layers, embed, ids, GROUPS, LQ, kb, vb, [1.0, 1.0, 1.0])
    for l in range(3):
        np.testing.assert_allclose(r["k_hat"][l], kd[l], rtol=0, atol=1e-9)
        np.testing.assert_allclose(r["v_hat"][l], vd[l], rtol=0, atol=1e-9)
    np.testing.assert_allclose(r["x_final"], xd[-LQ:], rtol=0, atol=1e-9)
    assert r["rows"] == [list(range(sum(GROUPS)))] * 3
    # no memory token recomputed anywhere: the memory-granularity path at ratio 0 (pinned to the re-rotated caches)
    r0 = ko.keep_prefill_tokens(sh, layers, embed, ids, GROUPS, LQ, kb, vb, [0.0, 0.0, 0.0])
    g0 = ko.keep_prefill(sh, layers, embed, ids, GROUPS, LQ, kb, vb, [0.0, 0.0, 0.0], 1)
    for l in range(3):
        assert np.array_equal(r0["k_hat"][l], g0["k_hat"][l]) and np.array_equal(r0["v_hat"][l], g0["v_hat"][l])
    assert np.array_equal(r0["x_final"], g0["x_final"]) and r0["rows"] == [[], [], []]


def test_whole_memories_forced_equals_the_memory_granularity_path():
    """Token rows that happen to be whole memories: the token path must do exactly what the (independently
    pinned) memory path does when forced to those memories."""
    shape, (sh, layers, embed, ids, kb, vb) = _problem(seed=3)
    sets = [[0, 1, 2, 3], [1, 3], [3]]
    off = ko.group_offsets(GROUPS)
    rows = [[int(p) for g in s for p in range(off[g], off[g + 1])] for s in sets]
    g = ko.keep_prefill(sh, layers, embed, ids, GROUPS, LQ, kb, vb, [1.0, 0.5, 0.25], 2, forced_sets=sets)
    t = ko.keep_prefill_tokens(sh, layers, embed, ids, GROUPS, LQ, kb, vb, [1.0, 0.5, 0.25], forced_rows=rows)
    for l in range(3):
        np.testing.assert_allclose(t["k_hat"][l], g["k_hat"][l], rtol=0, atol=1e-12)
        np.testing.assert_allclose(t["v_hat"][l], g["v_hat"][l], rtol=0, atol=1e-12)
    np.testing.assert_allclose(t["x_final"], g["x_final"], rtol=0, atol=1e-12)


def test_deviation_vanishes_where_the_cache_is_already_right():
    """Layer 0's K/V depend on the token alone, and nothing precedes the first memory: both are cached exactly,
    so their deviation is zero (rounding only); a later memory that attends to earlier ones deviates."""
    shape, (sh, layers, embed, ids, kb, vb) = _problem(seed=5)
    r = ko.keep_prefill_tokens(sh, layers, embed, ids, GROUPS, LQ, kb, vb, [1.0, 1.0, 1.0])
    scale = max(float(d.max()) for d in r["deviation"][1:])
    assert scale > 1e-6
    assert r["deviation"][0].max() < 1e-20 * max(1.0, scale) + 1e-20
    for l in (1, 2):
        assert r["deviation"][l][:GROUPS[0]].max() < 1e-20          # first memory
        assert r["deviation"][l][GROUPS[0]:].min() > 0              # every later token has changed


def test_deviation_closed_form():
    rng = np.random.default_rng(2)
    k_old = rng.standard_normal((6, 2, 4))
    v_old = rng.standard_normal((6, 2, 4))
    dk = np.zeros_like(k_old)
    dv = np.zeros_like(v_old)
    dk[1, 0, 2] = 3.0                 # one coordinate moved by 3 -> 9
    dv[2, 1, :] = 0.5                 # four coordinates moved by 1/2 -> 1
    dk[3, :, :] = 1.0
    dv[3, :, :] = -1.0                # all 8 + 8 coordinates moved by 1 -> 16
    d = ko.token_deviation(k_old + dk, v_old + dv, k_old, v_old)
    np.testing.assert_allclose(d, [0.0, 9.0, 1.0, 16.0, 0.0, 0.0], rtol=0, atol=1e-12)


def test_select_tokens_brute_force_and_ties():
    rng = np.random.default_rng(7)
    for trial in range(200):
        n = int(rng.integers(1, 8))
        dev = rng.integers(0, 4, size=n).astype(np.float64) if trial % 2 else rng.random(n)
        for k in range(0, n + 1):
            got = ko.select_tokens(dev, k)
            assert got == sorted(got) and len(got) == k
            # brute force: among all k-subsets, the one whose sorted (value desc, index asc) key list is smallest
            best = min(itertools.combinations(range(n), k),
                       key=lambda c: sorted((-float(np.float32(dev[i])), i) for i in c))
            assert got == list(best)
    assert ko.select_tokens(np.array([1.0, 2.0, 2.0, 2.0, 0.5]), 2) == [1, 2]      # lower index wins a tie
    # values that differ only beyond binary32 are equal for the selection
    assert ko.select_tokens(np.array([1.0, 1.0 + 1e-12]), 1) == [0]


def test_budget_nesting_and_sizes():
    shape, (sh, layers, embed, ids, kb, vb) = _problem(seed=9, n_layers=4)
    n_mem = sum(GROUPS)
    ratios = [1.0, 1.0, 0.5, 0.2]
    r = ko.keep_prefill_tokens(sh, layers, embed, ids, GROUPS, LQ, kb, vb, ratios)
    assert [len(x) for x in r["rows"]] == [n_mem, n_mem, 12, 5]          # ceil(0.5 * 24), ceil(0.2 * 24)
    for a, b in zip(r["rows"], r["rows"][1:]):
        assert set(b) <= set(a) and b == sorted(b)
    # the kept tokens are the top of layer 1's deviation
    want = ko.select_tokens(r["deviation"][1], 12)
    assert r["rows"][2] == [r["rows"][1][i] for i in want]
    assert ko.token_budget_count(0.1, 32768, 40000) == 3277 and ko.token_budget_count(np.float32(0.1), 10, 10) == 1
    assert ko.token_budget_count(0.0, 100, 50) == 0 and ko.token_budget_count(1.0, 100, 50) == 50


def test_recomputed_tokens_are_written_in_place_and_the_rest_is_the_loaded_cache():
    shape, (sh, layers, embed, ids, kb, vb) = _problem(seed=11)
    rows = [list(range(sum(GROUPS))), [6, 7, 15, 20], [7, 20]]
    t = ko.keep_prefill_tokens(sh, layers, embed, ids, GROUPS, LQ, kb, vb, [1.0, 0.2, 0.1], forced_rows=rows)
    for l in (1, 2):
        kh, vh = ko.realign_concat(sh, kb[l], vb[l], GROUPS, LQ)
        untouched = [p for p in range(sum(GROUPS)) if p not in rows[l]]
        assert np.array_equal(t["k_hat"][l][untouched], kh[untouched]) and np.array_equal(t["v_hat"][l][untouched], vh[untouched])
        assert not np.allclose(t["k_hat"][l][rows[l]], kh[rows[l]])
