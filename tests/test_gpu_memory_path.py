"""GPU parity of the memory-update path (Section 4.1): a unit's KV computed on its own through the
C ABI against the oracle's dense prefill of that unit, and the whole loop
store -> stale units -> unit caches -> joined prompt -> selective prefill against the oracle's."""
import numpy as np
import pytest
import torch

import keep_synth as ks
from oracle import keep_oracle as ko
from oracle.memory_oracle import MemoryOracle
from gpu_util import Problem, max_rel, to_np
from paper_2602_23592_amd import KeepMemory, KeepPrompt

pytestmark = pytest.mark.gpu

F32 = ks.ModelShape(2, 128, 6, 2, 64, 200, 211, 1.0e6, 1e-6, "f32")
BF16 = ks.ModelShape(2, 512, 8, 2, 128, 1024, 509, 1.0e6, 1e-6, "bf16")


def unit_cache(ctx, shape, tokens):
    dt = ks.torch_dtype(shape.storage)
    k = torch.empty((shape.n_layers, len(tokens), shape.n_kv_heads, shape.head_dim), dtype=dt, device="cuda")
    v = torch.empty_like(k)
    ctx.precompute_group(tokens, k, v)
    return k, v


@pytest.mark.parametrize("shape,tol", [(F32, 1e-4), (BF16, 2e-2)], ids=["f32", "bf16_mfma"])
def test_unit_cache_matches_dense_prefill_of_the_unit(shape, tol):
    pb = Problem(shape, [1], 1, seed=2, std=0.08, bias=True)          # weights and embedding only
    ctx = pb.context(max_tokens=520, max_groups=4)
    rng = np.random.default_rng(9)
    for n in (1, 2, 33, 64, 200, 513):
        tokens = [int(t) for t in rng.integers(0, shape.vocab, size=n)]
        k, v = unit_cache(ctx, shape, tokens)
        torch.cuda.synchronize()
        kr, vr, _ = ko.dense_prefill(pb.sh, pb.layers, pb.embed, np.asarray(tokens))
        for l in range(shape.n_layers):
            ek, ev = max_rel(to_np(k[l]), kr[l]), max_rel(to_np(v[l]), vr[l])
            print(shape.storage, n, l, "K %.2e V %.2e" % (ek, ev))
            assert ek < tol and ev < tol, (n, l)


def test_unit_cache_error_paths():
    pb = Problem(F32, [1], 1, seed=2)
    ctx = pb.context(max_tokens=16, max_groups=1)
    from paper_2602_23592_amd import KeepError
    k = torch.empty((2, 32, 2, 64), device="cuda")
    with pytest.raises(KeepError):
        ctx.precompute_group(list(range(32)), k, k.clone())          # above max_tokens
    with pytest.raises(KeepError):
        ctx.precompute_group([F32.vocab], k, k.clone())              # token outside the vocabulary


def test_update_loop_end_to_end_fp32():
    """Three rounds of memory updates with a window of 2 steps.  After each round both sides compute
    the stale units' caches (library on the GPU, oracle on the CPU), keep the others, join all units
    with an instruction and run the selective prefill; caches, final rows and sets must agree."""
    shape = F32
    pb = Problem(shape, [1], 1, seed=4, std=0.1, bias=True)
    ctx = pb.context(max_tokens=400, max_groups=16)
    lib_mem, ora = KeepMemory(2), MemoryOracle(2)
    rng = np.random.default_rng(21)
    tok = lambda n: [int(t) for t in rng.integers(0, shape.vocab, size=n)]
    instr = tok(9)
    rounds = [
        [("put", 0, 0, tok(17)), ("put", 0, 1, tok(30)), ("put", 0, 2, tok(5)), ("put", 1, 10, tok(40)), ("put", 1, 11, tok(8))],
        [("put", 1, 10, tok(33))],
        [],                                     # group 0 has been quiet for 2 steps: becomes one static unit
        [("put", 2, 20, tok(12))],
        [("put", 0, 1, tok(21))],              # hits the static group: back to per-segment units
    ]
    gpu_cache, cpu_cache = {}, {}               # (kind, id) -> caches
    seen_static = False
    for r, ops in enumerate(rounds):
        for _, g, s, t in ops:
            assert lib_mem.put(g, s, t) == ora.put(g, s, t)
        rep, to_dyn, to_sta = lib_mem.end_step()
        orep = ora.end_step()
        assert (rep.dirty_units, rep.dirty_tokens, to_dyn, to_sta) == \
               (orep.dirty_units, orep.dirty_tokens, orep.to_dynamic, orep.to_static)
        units, ounits = lib_mem.units(), ora.units()
        assert [(u.kind, u.id, u.n_tokens, u.dirty) for u in units] == \
               [(u.kind, u.ident, u.n_tokens, int(u.dirty)) for u in ounits]
        seen_static |= any(u.kind == 0 for u in units)
        glen, kinds, ids = [], [], []
        for i, (u, ou) in enumerate(zip(units, ounits)):
            key = (u.kind, u.id)
            tokens = lib_mem.unit_tokens(i, u.n_tokens)
            assert tokens == ora.unit_tokens(ou)
            if u.dirty:
                gpu_cache[key] = unit_cache(ctx, shape, tokens)
                kr, vr, _ = ko.dense_prefill(pb.sh, pb.layers, pb.embed, np.asarray(tokens))
                cpu_cache[key] = (kr, vr)
                lib_mem.mark_computed(i)
                ora.mark_computed(ou)
            glen.append(u.n_tokens); kinds.append(u.kind); ids += tokens
        ids = np.asarray(ids + instr, dtype=np.int32)
        G, L = len(glen), shape.n_layers
        keys = [(u.kind, u.id) for u in units]
        kb_d = [[gpu_cache[k][0][l] for k in keys] for l in range(L)]
        vb_d = [[gpu_cache[k][1][l] for k in keys] for l in range(L)]
        pr = KeepPrompt(glen, len(instr), ids, kb_d, vb_d, L, 0, kinds)
        ratios = [1.0, 0.5]
        n = sum(glen) + len(instr)
        kc = torch.empty((L, n, shape.n_kv_heads, shape.head_dim), device="cuda")
        vc = torch.empty_like(kc)
        xf = torch.empty((len(instr), shape.hidden), device="cuda")
        sets, _ = ctx.prefill(pr, ratios, 2, kc, vc, xf)
        torch.cuda.synchronize()
        kb = [[cpu_cache[k][0][l] for k in keys] for l in range(L)]
        vb = [[cpu_cache[k][1][l] for k in keys] for l in range(L)]
        ref = ko.keep_prefill(pb.sh, pb.layers, pb.embed, ids, glen, len(instr), kb, vb, ratios, 2)
        print("round", r, "units", [(u.kind, u.id, u.n_tokens) for u in units], "sets", sets)
        assert sets == ref["sets"]
        for l in range(L):
            assert max_rel(to_np(kc[l]), ref["k_hat"][l]) < 1e-4
            assert max_rel(to_np(vc[l]), ref["v_hat"][l]) < 1e-4
        assert max_rel(to_np(xf), ref["x_final"]) < 1e-4
    assert seen_static


@pytest.mark.parametrize("shape,tol", [(F32, 1e-4), (BF16, 2e-2)], ids=["f32", "bf16_mfma"])
def test_units_cached_in_one_pass_match_each_unit_alone(shape, tol):
    """Several units through keep_precompute_groups: every unit's blocks against the oracle's dense prefill of
    that unit on its own (local positions, attention inside the unit only).  Lengths straddle the 64-key tiles
    and the query tiles of the kernels."""
    pb = Problem(shape, [1], 1, seed=2, std=0.05, bias=True)
    lens = [1, 33, 64, 65, 200, 7, 130, 2, 300]
    total = sum(lens)
    ctx = pb.context(max_tokens=total, max_groups=4)
    rng = np.random.default_rng(13)
    tokens = [int(t) for t in rng.integers(0, shape.vocab, size=total)]
    dt = ks.torch_dtype(shape.storage)
    k = torch.empty((shape.n_layers, total, shape.n_kv_heads, shape.head_dim), dtype=dt, device="cuda")
    v = torch.empty_like(k)
    ctx.precompute_groups(lens, tokens, k, v)
    torch.cuda.synchronize()
    off = 0
    for n in lens:
        kr, vr, _ = ko.dense_prefill(pb.sh, pb.layers, pb.embed, np.asarray(tokens[off:off + n]))
        for l in range(shape.n_layers):
            ek = max_rel(to_np(k[l, off:off + n]), kr[l])
            ev = max_rel(to_np(v[l, off:off + n]), vr[l])
            assert ek < tol and ev < tol, (n, l, ek, ev)
        off += n
    # the next ordinary call is back to whole-prompt attention and global positions
    k1, v1 = unit_cache(ctx, shape, tokens[:40])
    kr, vr, _ = ko.dense_prefill(pb.sh, pb.layers, pb.embed, np.asarray(tokens[:40]))
    assert max_rel(to_np(k1[-1]), kr[-1]) < tol and max_rel(to_np(v1[-1]), vr[-1]) < tol


def test_fused_projection_epilogue_with_unit_local_positions():
    """Enough rows for the 256 x 256 GEMM tiles, whose QKV projection carries bias, RoPE and the K/V scatter in its
    epilogue (with tiles of the last round cut along K, which take the separate fix-up kernel): several units
    cached in one pass, so that the rotation uses the unit-local position (cache row minus the unit's first row),
    two layers, biases on; every unit's blocks against the oracle's dense prefill of that unit alone."""
    shape = ks.ModelShape(2, 2048, 16, 4, 128, 2048, 311, 1.0e6, 1e-6, "bf16")
    pb = Problem(shape, [1], 1, seed=5, std=0.03, bias=True)
    lens = [700, 1024, 513, 64, 900, 1100, 300, 777, 1000, 652]          # 7030 rows: 28 row tiles x 12 column tiles
    total = sum(lens)
    ctx = pb.context(max_tokens=total, max_groups=4)
    assert ctx.uses_mfma
    rng = np.random.default_rng(17)
    tokens = [int(t) for t in rng.integers(0, shape.vocab, size=total)]
    k = torch.full((shape.n_layers, total, shape.n_kv_heads, shape.head_dim), float("nan"), dtype=torch.bfloat16, device="cuda")
    v = k.clone()
    ctx.precompute_groups(lens, tokens, k, v)
    torch.cuda.synchronize()
    assert not torch.isnan(k).any() and not torch.isnan(v).any()
    off = 0
    for n in lens:
        kr, vr, _ = ko.dense_prefill(pb.sh, pb.layers, pb.embed, np.asarray(tokens[off:off + n]))
        for l in range(shape.n_layers):
            ek = max_rel(to_np(k[l, off:off + n]), kr[l])
            ev = max_rel(to_np(v[l, off:off + n]), vr[l])
            assert ek < 2e-2 and ev < 2e-2, (n, l, ek, ev)
        off += n
