"""keep_select_groups_static (the entry point for callers that cannot allocate) against keep_select_groups.

Both run the same selection kernel; the static one keeps its scratch (candidate lengths, their total) in a
device array built into the library and takes inputs and outputs in caller-allocated device memory.  Integer
results: bit-exact.  Two calls in a row share the array, the second with a smaller input."""
import numpy as np
import pytest
import torch

import keep_synth as ks
from gpu_util import Problem

pytestmark = pytest.mark.gpu


def _case(rng, G, m, ties=False, empty_query=False):
    glen = [int(v) for v in rng.integers(1, 50, size=G)]
    groups = sorted(rng.choice(G, size=m, replace=False).tolist())
    S = np.tril(rng.random((m + 1, m)), -1).astype(np.float32)
    S[m] = rng.random(m).astype(np.float32)
    if ties:
        S = (np.round(S * 4) / 4).astype(np.float32)
    if empty_query:
        S[m] = 0.0
    return glen, groups, S


def test_static_selection_equals_the_context_selection():
    from paper_2602_23592_amd import binding as kb
    shape = ks.ModelShape(2, 64, 4, 2, 16, 96, 97, 1.0e4, 1e-6, "f32")
    pb = Problem(shape, [4] * 8, 2, seed=2, random_cache=True)
    ctx = pb.context(max_groups=1300)
    rng = np.random.default_rng(77)
    # pairs of calls in a row, the second smaller than the first (it must not see the first one's leftovers)
    sizes = [(1200, 1100), (40, 7), (300, 300), (64, 1), (33, 5), (9, 9), (500, 20), (12, 3)]
    dev = "cuda"
    n_checked = 0
    for pair_i, (m_big, m_small) in enumerate(sizes):
        for mode in (kb.KEEP_BUDGET_GROUP_COUNT, kb.KEEP_BUDGET_TOKENS):
            for sources in (kb.KEEP_SOURCES_QUERY_AND_SET, kb.KEEP_SOURCES_SET_ONLY):
                ctx.set_option(kb.KEEP_OPT_PROPAGATION_SOURCES, sources)
                calls = []
                for m in (m_big, m_small):
                    G = m + int(rng.integers(0, 9))
                    glen, groups, S = _case(rng, G, m, ties=(pair_i % 3 == 0), empty_query=(pair_i == 4))
                    # ratios that keep some, all (1.0) and none (0.0) of the candidates
                    ratio = [float(np.float32(rng.random())), 1.0, 0.0, float(np.float32(rng.random() * 0.3))][n_checked % 4]
                    hops = int(rng.integers(1, 5))
                    want, want_runs = ctx.select_groups(S, groups, glen, ratio, hops, mode)
                    # device inputs and the output buffer: allocated here, before the calls under test
                    S_d = torch.from_numpy(S).to(dev).contiguous()
                    g_d = torch.tensor(groups, dtype=torch.int32, device=dev)
                    l_d = torch.tensor(glen, dtype=torch.int32, device=dev)
                    res = torch.full((m + 2,), -7, dtype=torch.int32, device=dev)
                    calls.append((S_d, g_d, l_d, sum(glen), ratio, hops, res, want, want_runs))
                    n_checked += 1
                torch.cuda.synchronize()
                for S_d, g_d, l_d, n_mem, ratio, hops, res, _, _ in calls:      # two calls in a row, no sync between
                    kb.select_groups_static(S_d, g_d, l_d, n_mem, ratio, hops, mode, sources, res)
                torch.cuda.synchronize()
                for S_d, g_d, l_d, n_mem, ratio, hops, res, want, want_runs in calls:
                    out = res.cpu().numpy()
                    got = [int(v) for v in out[2:2 + out[0]]]
                    assert got == want and int(out[1]) == want_runs, (pair_i, mode, sources, ratio, hops, got, want)
    assert n_checked == len(sizes) * 2 * 2 * 2


def test_static_selection_argument_errors():
    from paper_2602_23592_amd import binding as kb
    dev = "cuda"
    m = 5
    S = torch.zeros((m + 1) * m, dtype=torch.float32, device=dev)
    g = torch.arange(m, dtype=torch.int32, device=dev)
    gl = torch.full((m,), 3, dtype=torch.int32, device=dev)
    res = torch.zeros(m + 2, dtype=torch.int32, device=dev)

    def status(**kw):
        args = dict(S=S, groups=g, group_len=gl, mem_tokens=15, ratio_next=0.5, hops=2, budget_mode=0,
                    propagation_sources=0, result=res)
        args.update(kw)
        with pytest.raises(kb.KeepError) as e:
            kb.select_groups_static(**args)
        return e.value.status

    assert status(hops=0) == kb.KEEP_ERR_INVALID_ARG
    assert status(ratio_next=1.5) == kb.KEEP_ERR_INVALID_ARG
    assert status(budget_mode=3) == kb.KEEP_ERR_INVALID_ARG
    assert status(propagation_sources=2) == kb.KEEP_ERR_INVALID_ARG
    assert status(mem_tokens=2) == kb.KEEP_ERR_INVALID_ARG
    # more candidates than the static scratch holds: refused on the host, nothing is launched
    big = 4097
    lib = kb.load_library()
    st = lib.keep_select_groups_static(S.data_ptr(), g.data_ptr(), big, gl.data_ptr(), big, big, 0.5, 2, 0, 0,
                                       res.data_ptr(), None)
    assert st == kb.KEEP_ERR_WORKSPACE
    assert b"4096" in lib.keep_last_error(None)
    # and a good call still works afterwards
    kb.select_groups_static(S, g, gl, 15, 0.5, 2, 0, 0, res)
    torch.cuda.synchronize()
    assert int(res[0]) == 3
