"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element."""
import math

import numpy as np
import pytest
import torch

import keep_synth as ks
from oracle import keep_oracle as ko
from gpu_util import Problem, max_rel, to_np, update_err, layer_state_err

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}     # max |a-b| / max |b| per tensor, per layer


def _tiny_problem():
    w = ks.workload("tiny")
    glen, _ = ks.group_lengths(w)
    return w, Problem(w.shape, glen, w.instr_len, seed=0, std=0.02, bias=False, embed_scale=0.02)


def test_tiny_prefill_fp32_end_to_end():
    w, pb = _tiny_problem()
    ratios = ks.ratio_schedule(w.ratio, w.shape.n_layers)
    ref = ko.keep_prefill(pb.sh, pb.layers, pb.embed, pb.ids, pb.group_len, pb.instr_len, pb.kb, pb.vb,
                          [float(r) for r in ratios], w.hops)
    ctx, pr = pb.context(), pb.prompt()
    kc, vc = pb.empty_cache()
    xf = torch.empty((pb.instr_len, w.shape.hidden), dtype=torch.float32, device="cuda")
    sets, rep = ctx.prefill(pr, ratios, w.hops, kc, vc, xf, want_report=True)
    torch.cuda.synchronize()
    print("sets", sets, "oracle", ref["sets"], "ms", rep.ms_total)
    assert sets == ref["sets"]
    for l in range(w.shape.n_layers):
        assert max_rel(to_np(kc[l]), ref["k_hat"][l]) < TOL["f32"]
        assert max_rel(to_np(vc[l]), ref["v_hat"][l]) < TOL["f32"]
    assert max_rel(to_np(xf), ref["x_final"]) < TOL["f32"]
    assert not torch.isnan(kc).any() and not torch.isnan(vc).any()
    # behind the last layer only the instruction's rows are read: its output projection and FFN ran on those
    last = w.shape.n_layers - 1
    assert rep.rows[last] > pb.instr_len and rep.ffn_rows[last] == pb.instr_len


SHAPES = {
    "f32_small": ks.ModelShape(2, 64, 4, 2, 16, 96, 97, 1.0e4, 1e-6, "f32"),
    "bf16_small_generic": ks.ModelShape(2, 64, 4, 2, 16, 96, 97, 1.0e4, 1e-6, "bf16"),
    "f32_dh64": ks.ModelShape(2, 128, 6, 2, 64, 200, 211, 1.0e6, 1e-6, "f32"),
}
LAYOUTS = [
    ([1, 31, 33, 64, 65], 7),
    ([5], 1),
    ([3, 1, 1, 9], 1),
    ([17, 40, 2, 129], 33),
]


@pytest.mark.parametrize("shape_name", list(SHAPES))
@pytest.mark.parametrize("layout", LAYOUTS)
def test_layer_teacher_forced(shape_name, layout):
    """One layer given the oracle's set and the oracle's input rows: K/V cache, output rows, scores."""
    shape = SHAPES[shape_name]
    glen, lq = layout
    pb = Problem(shape, glen, lq, seed=3, std=0.1, bias=True)
    ctx, pr = pb.context(), pb.prompt()
    G = len(glen)
    tol = TOL[shape.storage]
    rng = np.random.default_rng(5)
    for layer, groups in ((0, list(range(G))), (1, sorted(rng.choice(G, size=max(1, G // 2), replace=False).tolist())),
                          (1, [])):
        n_rows = pr.n_rows(groups)
        x_t = ks.make_random_rows(n_rows, shape.hidden, shape.storage, seed=11 + layer)
        x_np = ks.to_numpy_f64(x_t)
        kh, vh = pb.oracle_joined_cache(layer)
        probe = {}
        xo_ref, lse_ref, S_ref = ko.selective_layer(pb.sh, pb.layers[layer], x_np, groups, glen, lq, kh, vh, probe=probe)
        kc, vc = pb.empty_cache(1)
        x_out = torch.empty_like(x_t, device="cuda")
        ctx.recompute_layer(pr, layer, groups, x_t.cuda(), x_out, kc[0], vc[0])
        eo, el = layer_state_err(ctx, n_rows, probe, lse_ref)
        nxt, runs, S = ctx.score_groups(pr, layer, groups, 0.5, 2)
        torch.cuda.synchronize()
        assert max_rel(to_np(kc[0]), kh) < tol, (layer, groups)
        assert max_rel(to_np(vc[0]), vh) < tol
        assert max_rel(to_np(x_out), xo_ref) < tol
        # the attention output and its log-sum-exp on their own scale, and the layer's update without the
        # residual stream's cushion
        ed, allow = update_err(to_np(x_out), x_np, xo_ref, shape.storage)
        assert eo < tol and el < tol and ed < tol + allow, (layer, groups, eo, el, ed, allow)
        if len(groups):
            assert np.abs(S - S_ref).max() <= tol * max(S_ref.max(), 1e-30), (S, S_ref)
            # the device selection is the oracle's selection applied to the device's own scores
            want, want_runs = ko.select_multihop(S, groups, glen, 0.5, 2)
            assert nxt == want and runs == want_runs


def test_fixed_points_on_gpu():
    """Ratio 1 at every layer = dense causal prefill; ratio 0 = re-rotated concatenation."""
    shape = SHAPES["f32_dh64"]
    glen, lq = [20, 33, 7, 64], 9
    pb = Problem(shape, glen, lq, seed=1, std=0.1, bias=True)
    ctx, pr = pb.context(), pb.prompt()
    kd, vd, xd = ko.dense_prefill(pb.sh, pb.layers, pb.embed, pb.ids, 0)
    kc, vc = pb.empty_cache()
    xf = torch.empty((lq, shape.hidden), dtype=torch.float32, device="cuda")
    sets, _ = ctx.prefill(pr, [1.0, 1.0], 2, kc, vc, xf)
    assert sets == [[0, 1, 2, 3]] * 2
    for l in range(2):
        assert max_rel(to_np(kc[l]), kd[l]) < 1e-4 and max_rel(to_np(vc[l]), vd[l]) < 1e-4
    assert max_rel(to_np(xf), xd[-lq:]) < 1e-4
    sets, _ = ctx.prefill(pr, [0.0, 0.0], 2, kc, vc, xf)
    assert sets == [[], []]
    nm = sum(glen)
    for l in range(2):
        kh, vh = pb.oracle_joined_cache(l)
        assert max_rel(to_np(kc[l][:nm]), kh[:nm]) < 1e-6
        assert torch.equal(vc[l][:nm].cpu(), torch.from_numpy(vh[:nm]).float())    # values are copied bit for bit


def test_selection_bit_exact_against_oracle():
    shape = SHAPES["f32_small"]
    pb = Problem(shape, [4] * 40, 2, seed=2, random_cache=True)
    ctx = pb.context(max_groups=64)
    rng = np.random.default_rng(9)
    n_checked = 0
    for trial in range(60):
        G = int(rng.integers(2, 41))
        glen = [int(v) for v in rng.integers(1, 50, size=G)]
        m = int(rng.integers(1, G + 1))
        groups = sorted(rng.choice(G, size=m, replace=False).tolist())
        S = np.tril(rng.random((m + 1, m)), -1).astype(np.float32)
        S[m] = rng.random(m).astype(np.float32)
        if trial % 4 == 0:                      # ties
            S = (np.round(S * 4) / 4).astype(np.float32)
        if trial % 7 == 0:
            S[m] = 0.0                          # query attends to nothing
        for mode in (0, 1):
            for hops in (1, 2, 5):
                ratio = float(np.float32(rng.random()))
                want, runs = ko.select_multihop(S, groups, glen, ratio, hops, mode)
                got, got_runs = ctx.select_groups(S, groups, glen, ratio, hops, mode)
                assert got == want, (trial, mode, hops, ratio)
                assert got_runs == runs
                n_checked += 1
    assert n_checked == 360


def test_selection_literal_propagation_bit_exact_against_oracle():
    """KEEP_SOURCES_SET_ONLY: the propagation averages the rows of the relevant set alone (the section's wording
    taken literally).  Same bit-exact bar against the oracle's drop_query variant; the option is per context and
    can be switched back."""
    from paper_2602_23592_amd import binding as kbind
    shape = SHAPES["f32_small"]
    pb = Problem(shape, [4] * 40, 2, seed=2, random_cache=True)
    ctx = pb.context(max_groups=400)
    rng = np.random.default_rng(29)
    differs = 0
    for trial in range(40):
        G = int(rng.integers(2, 41)) if trial < 36 else int(rng.integers(260, 400))
        glen = [int(v) for v in rng.integers(1, 50, size=G)]
        m = int(rng.integers(1, G + 1))
        groups = sorted(rng.choice(G, size=m, replace=False).tolist())
        S = np.tril(rng.random((m + 1, m)), -1).astype(np.float32)
        S[m] = rng.random(m).astype(np.float32)
        if trial % 4 == 0:
            S = (np.round(S * 4) / 4).astype(np.float32)
        if trial % 7 == 0:
            S[m] = 0.0                          # empty first set: the literal variant has no source at all
        for mode in (0, 1):
            for hops in (2, 5):
                ratio = float(np.float32(rng.random()))
                ctx.set_option(kbind.KEEP_OPT_PROPAGATION_SOURCES, kbind.KEEP_SOURCES_SET_ONLY)
                want, runs = ko.select_multihop(S, groups, glen, ratio, hops, mode, drop_query=True)
                got, got_runs = ctx.select_groups(S, groups, glen, ratio, hops, mode)
                assert got == want and got_runs == runs, (trial, mode, hops, ratio)
                ctx.set_option(kbind.KEEP_OPT_PROPAGATION_SOURCES, kbind.KEEP_SOURCES_QUERY_AND_SET)
                want2, runs2 = ko.select_multihop(S, groups, glen, ratio, hops, mode)
                got2, got_runs2 = ctx.select_groups(S, groups, glen, ratio, hops, mode)
                assert got2 == want2 and got_runs2 == runs2
                differs += want != want2
    assert differs > 0          # the two readings do select differently on some of these matrices
    with pytest.raises(kbind.KeepError):
        ctx.set_option(kbind.KEEP_OPT_PROPAGATION_SOURCES, 7)
    with pytest.raises(kbind.KeepError):
        ctx.set_option(99, 0)


def test_selection_bit_exact_with_many_candidates():
    """The selector with hundreds to thousands of candidates: row totals over several row blocks and ragged
    column tiles, several candidates per thread, token-budget walks over long orders."""
    shape = SHAPES["f32_small"]
    pb = Problem(shape, [4] * 8, 2, seed=2, random_cache=True)
    ctx = pb.context(max_groups=1600)
    rng = np.random.default_rng(19)
    for m in (257, 300, 1100, 1500):
        G = m + 7
        glen = [int(v) for v in rng.integers(1, 50, size=G)]
        groups = sorted(rng.choice(G, size=m, replace=False).tolist())
        S = np.tril(rng.random((m + 1, m)), -1).astype(np.float32)
        S[m] = rng.random(m).astype(np.float32)
        if m == 300:
            S = (np.round(S * 8) / 8).astype(np.float32)      # many ties
        for mode in (0, 1):
            for hops, ratio in ((1, 0.1), (3, 0.07), (4, 0.3)):
                want, runs = ko.select_multihop(S, groups, glen, ratio, hops, mode)
                got, got_runs = ctx.select_groups(S, groups, glen, ratio, hops, mode)
                assert got == want, (m, mode, hops)
                assert got_runs == runs


def test_prefill_multi_layer_sets_and_token_budget():
    shape = ks.ModelShape(4, 64, 4, 2, 16, 96, 97, 1.0e4, 1e-6, "f32")
    glen, lq = [9, 14, 3, 22, 8, 17, 5, 12], 6
    pb = Problem(shape, glen, lq, seed=4, std=0.15, bias=True)
    ctx, pr = pb.context(), pb.prompt()
    ratios = [1.0, 0.75, 0.5, 0.25]
    for mode in (0, 1):
        ref = ko.keep_prefill(pb.sh, pb.layers, pb.embed, pb.ids, glen, lq, pb.kb, pb.vb, ratios, 3, mode)
        kc, vc = pb.empty_cache()
        xf = torch.empty((lq, shape.hidden), dtype=torch.float32, device="cuda")
        sets, rep = ctx.prefill(pr, ratios, 3, kc, vc, xf, budget_mode=mode, want_report=True)
        assert sets == ref["sets"], (mode, sets, ref["sets"])
        for l in range(4):
            assert max_rel(to_np(kc[l]), ref["k_hat"][l]) < 1e-4
            assert max_rel(to_np(vc[l]), ref["v_hat"][l]) < 1e-4
        assert max_rel(to_np(xf), ref["x_final"]) < 1e-4
        assert [rep.rows[l] for l in range(4)] == [sum(glen[g] for g in s) + lq for s in ref["sets"]]


def test_host_resident_kv_load_modes_are_identical():
    """Pinned-host group caches: serial / next-layer / layer-balanced loading give the same bits."""
    shape = ks.ModelShape(4, 64, 4, 2, 16, 96, 97, 1.0e4, 1e-6, "f32")
    glen, lq = [9, 14, 3, 22, 8, 17, 5, 12], 6
    pb = Problem(shape, glen, lq, seed=4, std=0.15, bias=True)
    ctx = pb.context()
    ratios = [1.0, 0.75, 0.5, 0.25]
    outs = []
    for pinned, mode in ((False, 2), (True, 0), (True, 1), (True, 2)):
        pr = pb.prompt(pinned_host=pinned)
        kc, vc = pb.empty_cache()
        xf = torch.empty((lq, shape.hidden), dtype=torch.float32, device="cuda")
        sets, rep = ctx.prefill(pr, ratios, 3, kc, vc, xf, load_mode=mode, want_report=True)
        outs.append((sets, kc.cpu(), vc.cpu(), xf.cpu()))
        if pinned:
            assert sum(rep.bytes_loaded[l] for l in range(4)) > 0
    for o in outs[1:]:
        assert o[0] == outs[0][0]
        assert torch.equal(o[1], outs[0][1]) and torch.equal(o[2], outs[0][2]) and torch.equal(o[3], outs[0][3])


def test_three_streams_give_the_same_result():
    """Compute / evaluation / loading on three separate streams (Section 5's pipeline)."""
    shape = ks.ModelShape(3, 64, 4, 2, 16, 96, 97, 1.0e4, 1e-6, "f32")
    glen, lq = [9, 14, 3, 22, 8, 17, 5, 12], 6
    pb = Problem(shape, glen, lq, seed=8, std=0.15, bias=True)
    ratios = [1.0, 0.6, 0.3]
    from paper_2602_23592_amd import KeepContext
    outs = []
    for separate in (False, True):
        streams = [torch.cuda.Stream() for _ in range(3)] if separate else [None] * 3
        ctx = KeepContext(shape, pb.layers_d, pb.embed_d, pb.n_tokens, len(glen), 0, *streams)
        pr = pb.prompt(pinned_host=True)
        kc, vc = pb.empty_cache()
        xf = torch.empty((lq, shape.hidden), dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        sets, _ = ctx.prefill(pr, ratios, 2, kc, vc, xf)
        torch.cuda.synchronize()
        outs.append((sets, kc.cpu(), vc.cpu(), xf.cpu()))
        ctx.close()
    assert outs[0][0] == outs[1][0]
    for i in (1, 2, 3):
        assert torch.equal(outs[0][i], outs[1][i])


def test_error_paths_with_a_live_context():
    from paper_2602_23592_amd import KeepError, KeepPrompt
    from paper_2602_23592_amd import binding as kbind
    shape = SHAPES["f32_small"]
    glen, lq = [5, 9, 4], 3
    pb = Problem(shape, glen, lq, seed=2, std=0.1)
    ctx, pr = pb.context(), pb.prompt()
    kc, vc = pb.empty_cache()
    xf = torch.empty((lq, shape.hidden), dtype=torch.float32, device="cuda")
    x = torch.zeros((pr.n_rows([0, 2]), shape.hidden), dtype=torch.float32, device="cuda")

    def status(fn):
        with pytest.raises(KeepError) as e:
            fn()
        return e.value.status

    # scores before the layer was computed, or for another set: STATE
    assert status(lambda: ctx.score_groups(pr, 0, [0, 2], 0.5, 1)) == kbind.KEEP_ERR_STATE
    ctx.recompute_layer(pr, 0, [0, 2], x, x.clone(), kc[0], vc[0])
    assert status(lambda: ctx.score_groups(pr, 0, [0, 1], 0.5, 1)) == kbind.KEEP_ERR_STATE
    assert status(lambda: ctx.score_groups(pr, 1, [0, 2], 0.5, 1)) == kbind.KEEP_ERR_STATE
    ctx.score_groups(pr, 0, [0, 2], 0.5, 1)                   # the matching call works
    # bad sets and layers: INVALID_ARG
    assert status(lambda: ctx.recompute_layer(pr, 0, [2, 0], x, x, kc[0], vc[0])) == kbind.KEEP_ERR_INVALID_ARG
    assert status(lambda: ctx.recompute_layer(pr, 0, [0, 3], x, x, kc[0], vc[0])) == kbind.KEEP_ERR_INVALID_ARG
    assert status(lambda: ctx.recompute_layer(pr, 2, [0], x, x, kc[0], vc[0])) == kbind.KEEP_ERR_INVALID_ARG
    # ratio schedules: first layer is all or nothing, later layers never grow
    assert status(lambda: ctx.prefill(pr, [0.5, 0.5], 1, kc, vc, xf)) == kbind.KEEP_ERR_INVALID_ARG
    assert status(lambda: ctx.prefill(pr, [0.0, 0.5], 1, kc, vc, xf)) == kbind.KEEP_ERR_INVALID_ARG
    assert status(lambda: ctx.prefill(pr, [1.0, 0.5], 0, kc, vc, xf)) == kbind.KEEP_ERR_INVALID_ARG
    # prompt larger than the workspace: WORKSPACE
    big = KeepPrompt([5, 9, 4, 300], lq, np.zeros(321, dtype=np.int32), None, None, shape.n_layers)
    assert status(lambda: ctx.prefill(big, [1.0, 0.5], 1, kc, vc, xf)) == kbind.KEEP_ERR_WORKSPACE
    # token ids outside the vocabulary, empty instruction
    bad_tok = KeepPrompt(glen, lq, np.full(21, 97, dtype=np.int32), pb.kb_d, pb.vb_d, shape.n_layers)
    assert status(lambda: ctx.prefill(bad_tok, [1.0, 0.5], 1, kc, vc, xf)) == kbind.KEEP_ERR_INVALID_ARG
    no_q = KeepPrompt(glen, 0, pb.ids[:18], pb.kb_d, pb.vb_d, shape.n_layers)
    assert status(lambda: ctx.prefill(no_q, [1.0, 0.5], 1, kc, vc, xf)) == kbind.KEEP_ERR_INVALID_ARG
    # the context still works after the errors
    sets, _ = ctx.prefill(pr, [1.0, 0.5], 2, kc, vc, xf)
    assert len(sets[1]) == 2
