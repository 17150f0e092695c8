"""Benchmark of the selective-KV-recompute prefill on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]

A step is one whole keep_prefill (every layer: re-alignment of cached groups, QKV of the
recomputed rows, sparse-row attention over the joined cache, group scores + multi-hop
selection, output projection and FFN) of one seeded synthetic prompt, with weights and
group KV caches already resident in HBM.  Prints ONE JSON line: TTFT per step, prefill
tokens/s, the roofline figures of the dominant kernel measured with HIP events on the
stream the kernel runs on, and the CPU oracle timed on the host cores on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E


TRAFFIC_JSON = os.path.join(ROOT, "profiles", "keep_prefill_qwen14b_32k_gate_up_traffic.json")
TRAFFIC_SOURCES = ("paper_2602_23592_amd/csrc/gemm_mfma.hip",)


def sources_sha16(paths=TRAFFIC_SOURCES):
    """Hash of the sources of the roofline kernel: a stored counter figure holds only for the kernel it was measured on."""
    import hashlib
    h = hashlib.sha256()
    for rel in paths:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def stored_traffic():
    """L2-miss bytes per gate/up launch from the two rocprofv3 --pmc runs summarised under profiles/ (written by
    bench_profile_summary.py), or None when the kernel's source has changed since they were made."""
    try:
        with open(TRAFFIC_JSON) as f:
            t = json.load(f)
    except (OSError, ValueError):
        return None, "no stored counter run"
    if t.get("sources_sha16") != sources_sha16():
        return None, "stored counter run is for another build of the kernel (%s)" % t.get("sources_sha16")
    return int(t["bytes_per_launch"]), "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, %s" % t.get("measured_at", "")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="qwen14b_32k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--schedule", default=None, help="ratio schedule: linear (default of the workload) or const")
    ap.add_argument("--ratio", type=float, default=None, help="mean recompute ratio (default: the workload's)")
    ap.add_argument("--budget", default=None, help="groups or tokens (default: the workload's)")
    ap.add_argument("--load-mode", type=int, default=2, help="0 serial, 1 next-layer, 2 layer-balanced")
    ap.add_argument("--layers-json", default=None, help="also write the per-layer timing report to this file")
    ap.add_argument("--random-cache", action="store_true",
                    help="random group caches instead of caches prefilled by the library (faster set-up)")
    ap.add_argument("--sparse-rows", type=int, default=0,
                    help="diagnostic: pure reuse (ratio 0 at every layer) with an instruction of this many rows, "
                         "the regime where the sparse-row attention is bound by reading the cache once")
    ap.add_argument("--decode-tokens", type=int, default=0,
                    help="instead of the prefill benchmark: prefill once, then time the first token and this many "
                         "greedy decode steps over the joined cache")
    ap.add_argument("--memory-update", action="store_true",
                    help="measure the cost of one memory update on the workload's model shape instead of the prefill")
    ap.add_argument("--int4", action="store_true",
                    help="with --decode-tokens / --memory-update: INT4 weight-only projections (the launches of at "
                         "most 48 rows read the 4-bit form; the bf16 weights are its expansion)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the extra keys of the default run (the count-budget reading of the same prompt, the "
                         "other workloads, the loading modes and the token-granularity pair on the host-resident one)")
    ap.add_argument("--granularity", default="groups", help="groups (the method) or tokens (the comparison scheme)")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of one line: recompute ratio 5/10/20/30 %% x hops 1-4 on the workload, one JSON line each")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="launch one device copy of this many MiB before the warm-up: the known-size "
                         "kernel that scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    return ap.parse_args()


class ProfilerGate:
    """Asks an attached rocprofv3 (if any) to collect only the warm-up + timed steps, so that its
    per-kernel averages cover the same launches as this script's own HIP-event timings.  Without
    a profiler the calls do nothing."""

    def __init__(self):
        self.lib = None
        try:
            import ctypes
            self.lib = ctypes.CDLL("librocprofiler-sdk-roctx.so")
            self.lib.roctxProfilerPause.argtypes = [ctypes.c_uint64]
            self.lib.roctxProfilerResume.argtypes = [ctypes.c_uint64]
        except OSError:
            self.lib = None

    def pause(self):
        if self.lib is not None:
            self.lib.roctxProfilerPause(0)

    def resume(self):
        if self.lib is not None:
            self.lib.roctxProfilerResume(0)


def precompute_group_caches(ctx, w, glen, ids, torch):
    """Group caches made by the library's own dense path on each unit alone, at unit-local positions
    (Section 4.1: every static group and every dynamic segment is cached on its own), all units in one
    batched pass."""
    s = w.shape
    L, n_mem = s.n_layers, int(np.sum(glen))
    dt = torch.bfloat16 if s.storage == "bf16" else torch.float32
    kb_all = torch.empty((L, n_mem, s.n_kv_heads, s.head_dim), dtype=dt, device="cuda")
    vb_all = torch.empty_like(kb_all)
    ctx.precompute_groups([int(n) for n in glen], ids[:n_mem], kb_all, vb_all)
    torch.cuda.synchronize()
    return kb_all, vb_all


def decode_bench(ctx, prompt, ratios, w, s, n_tokens, budget_mode, a, torch, dt):
    """First token and short greedy decoding after the joined prefill (Section 1: the planner's answer is
    a short action).  Per decoded token the path reads every layer's weights, the vocabulary projection and
    the whole joined cache once: an HBM-bound regime."""
    k = a.decode_tokens
    cap = n_tokens + k + 1
    kc = torch.empty((s.n_layers, cap, s.n_kv_heads, s.head_dim), dtype=dt, device="cuda")
    vc = torch.empty_like(kc)
    xf = torch.empty((w.instr_len, s.hidden), dtype=dt, device="cuda")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(11)
    fn = torch.ones(s.hidden, dtype=dt, device="cuda")
    lm = (0.02 * torch.randn((s.vocab, s.hidden), generator=gen, device="cuda")).to(dt)
    ctx.prefill(prompt, ratios, w.hops, kc, vc, xf, budget_mode, a.load_mode, cache_rows=cap)

    def timed(n_new):
        for _ in range(a.warmup):
            ctx.decode(fn, lm, xf[-1], kc, vc, n_tokens, n_new)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            toks = ctx.decode(fn, lm, xf[-1], kc, vc, n_tokens, n_new)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / a.steps, toks

    ms_first, _ = timed(1)
    ms_all, toks = timed(k + 1)
    ms_tok = (ms_all - ms_first) / k
    esz = 2 if s.storage == "bf16" else 4
    qd, kvd = s.n_q_heads * s.head_dim, s.n_kv_heads * s.head_dim
    n_w = s.hidden * (qd + 2 * kvd) + qd * s.hidden + 3 * s.hidden * s.ffn_dim
    # INT4 form: half a byte per weight + one 4-byte scale/zero word per 128 weights
    w_layer = n_w * esz if not a.int4 else n_w // 2 + n_w // 128 * 4
    head = s.vocab * s.hidden * esz
    cache = 2.0 * (n_tokens + k / 2.0) * kvd * esz
    bytes_tok = s.n_layers * (w_layer + cache) + head
    return {"metric": "greedy decode over the joined cache", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
            "context_tokens": n_tokens, "decoded_tokens": k, "first_token_ms": round(ms_first, 3),
            "ms_per_token": round(ms_tok, 3), "tokens_per_s": round(1e3 / ms_tok, 1),
            "bytes_per_token": int(bytes_tok), "hbm": {"bound": "hbm", "achieved": round(bytes_tok / (ms_tok * 1e-3) / 1e9, 1),
                                                       "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                                       "frac": round(bytes_tok / (ms_tok * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)},
            "first_token_gbs": round(head / (ms_first * 1e-3) / 1e9, 1), "dtype": s.storage,
            "weights": "int4 weight-only (group 128) for the projections, bf16 LM head" if a.int4 else s.storage,
            "data": "synthetic", "tokens": toks[:8]}


def memory_update_cost(ctx, w, torch, steps, warmup):
    """Cost of one memory update (Section 4.1) on this model shape: the KV computation that the
    static-dynamic store asks for after (a) an update of one dynamic segment, (b) a static group that
    turned dynamic (each segment on its own), (c) a dynamic group that turned static (jointly)."""
    s = w.shape
    dt = torch.bfloat16 if s.storage == "bf16" else torch.float32
    seg, nseg = 64, 16
    rng = np.random.default_rng(3)
    toks = rng.integers(0, s.vocab, size=seg * nseg).astype(np.int32)
    k1 = torch.empty((s.n_layers, seg, s.n_kv_heads, s.head_dim), dtype=dt, device="cuda")
    v1 = torch.empty_like(k1)
    kg = torch.empty((s.n_layers, seg * nseg, s.n_kv_heads, s.head_dim), dtype=dt, device="cuda")
    vg = torch.empty_like(kg)

    def one_segment():
        ctx.precompute_group(toks[:seg], k1, v1)

    def every_segment():
        for i in range(nseg):
            ctx.precompute_group(toks[i * seg:(i + 1) * seg], k1, v1)

    def every_segment_one_pass():
        ctx.precompute_groups([seg] * nseg, toks, kg, vg)

    def whole_group():
        ctx.precompute_group(toks, kg, vg)

    def unit_of(n):
        ku = torch.empty((s.n_layers, n, s.n_kv_heads, s.head_dim), dtype=dt, device="cuda")
        vu = torch.empty_like(ku)
        return lambda: ctx.precompute_group(toks[:n], ku, vu)

    out = {}
    cases = [("dynamic_segment_update", one_segment, seg),
             ("static_to_dynamic_one_by_one", every_segment, seg * nseg),
             ("static_to_dynamic", every_segment_one_pass, seg * nseg),
             ("dynamic_to_static", whole_group, seg * nseg)]
    # one unit of n tokens: launches of a few rows stream the weights (at most 16 rows of bf16 weights, at most
    # 48 of the 4-bit form if it is attached), longer ones run on the matrix-core kernels with the bf16 weights
    cases += [("unit_%d_tokens" % n, unit_of(n), n) for n in (16, 32, 33, 48, 64, 65, 96, 128, 256, 512)]
    for name, fn, ntok in cases:
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        out[name] = {"ms": round(ms, 3), "tokens": ntok, "tokens_per_s": round(ntok / (ms * 1e-3), 1)}
    return {"metric": "memory update cost (KV computation the static-dynamic store triggers)",
            "segment_tokens": seg, "segments_per_group": nseg, "layers": s.n_layers, "n_gpus": 1,
            "steps": steps, "warmup": warmup, "dtype": s.storage, "data": "synthetic", "cases": out}


def visible_keys(sets, glen, lq):
    """sum over recomputed rows of (position + 1), per layer: the attention's key count."""
    off = np.concatenate([[0], np.cumsum(glen)]).astype(np.int64)
    n_mem = int(off[-1])
    out = []
    for st in sets:
        tot = 0
        for g in st:
            a, b = int(off[g]), int(off[g + 1])
            tot += (a + 1 + b) * (b - a) // 2
        a, b = n_mem, n_mem + lq
        tot += (a + 1 + b) * (b - a) // 2
        out.append(tot)
    return out


def cpu_baseline(w, glen, rows_per_layer, n_tokens):
    """The CPU oracle as it stands, timed on a bounded sample: one selective layer of this
    workload (layer 1, seeded random set of the layer's budget, random-draw caches and
    hidden rows), K/V refresh of all its rows, attention + projections + FFN of 256 and of
    768 sampled rows.  Whole-prefill tokens/s is extrapolated by row count."""
    import keep_synth as ks
    from oracle import keep_oracle as ko
    s = w.shape
    sh = ko.Shape(s.n_layers, s.hidden, s.n_q_heads, s.n_kv_heads, s.head_dim, s.ffn_dim, s.vocab, s.rope_theta,
                  s.rms_eps, s.storage)
    G = len(glen)
    ratios = ks.ratio_schedule(w.ratio, s.n_layers, w.schedule)
    rng = np.random.Generator(np.random.PCG64(5))
    if w.budget == "tokens":        # a seeded random set that fills the layer's token budget
        left, groups = ko.budget_tokens(float(ratios[1]), int(np.sum(glen))), []
        for g in rng.permutation(G):
            if glen[g] <= left:
                groups.append(int(g))
                left -= int(glen[g])
        groups.sort()
    else:
        groups = sorted(rng.choice(G, size=ko.budget_count(float(ratios[1]), G, G), replace=False).tolist())
    lw = {kk: (None if v is None else ks.to_numpy_f64(v)) for kk, v in ks.make_layer_weights(s, 1, "cpu").items()}
    kb, vb = ks.make_random_group_cache(s, glen, 1, seed=7)
    kb = [ks.to_numpy_f64(t) for t in kb]
    vb = [ks.to_numpy_f64(t) for t in vb]
    glist = [int(v) for v in glen]
    kh, vh = ko.realign_concat(sh, kb, vb, glist, w.instr_len)
    n_l = sum(glist[g] for g in groups) + w.instr_len
    x = ks.to_numpy_f64(ks.make_random_rows(n_l, s.hidden, s.storage, seed=11))
    times = []
    for n_s in (256, 768):
        pick = np.sort(rng.choice(n_l, size=min(n_s, n_l), replace=False))
        t0 = time.perf_counter()
        ko.selective_layer(sh, lw, x, groups, glist, w.instr_len, kh.copy(), vh.copy(), want_scores=False,
                           only_rows=pick)
        times.append(time.perf_counter() - t0)
    per_row = max((times[1] - times[0]) / 512.0, 1e-9)
    fixed = max(times[0] - 256 * per_row, 0.0)
    row_cost = per_row + fixed / n_l
    total_rows = int(np.sum(rows_per_layer))
    est = total_rows * row_cost
    cores = len(os.sched_getaffinity(0))
    threads = int(os.environ.get("OMP_NUM_THREADS", cores))
    return {"value": n_tokens / est, "unit": "tokens/s", "cores": min(cores, threads), "kind": "oracle",
            "sample": "oracle selective_layer, layer 1 of %d, %d rows over the %d-token cache: K/V refresh of all rows "
                      "+ attention/FFN of 256 and 768 sampled rows (%.1f s + %.1f s); whole prefill extrapolated by "
                      "row count (%d rows over all layers)" % (s.n_layers, n_l, n_tokens, times[0], times[1], total_rows),
            "seconds": times[0] + times[1], "extrapolated": True}


class Case:
    """One workload set up on the GPU: weights, context, prompt with its group caches, output buffers."""

    def __init__(self, name, a, torch, ks, kb, ratio=None, sparse_rows=0, layers=None, int4=False, random_cache=False,
                 extra_tokens=0):
        import dataclasses
        from paper_2602_23592_amd import KeepContext, KeepPrompt
        t0 = time.perf_counter()
        w = ks.workload(name)
        if ratio is not None:
            w = dataclasses.replace(w, ratio=ratio)
        if sparse_rows > 0:
            w = dataclasses.replace(w, instr_len=sparse_rows, ratio=0.0)
        self.w, self.s = w, w.shape
        s = w.shape
        self.torch, self.kb = torch, kb
        self.dt = torch.bfloat16 if s.storage == "bf16" else torch.float32
        self.glen, self.kinds = ks.group_lengths(w)
        self.G, self.lq = len(self.glen), w.instr_len
        self.n_tokens = w.mem_tokens + self.lq
        self.layers4 = None
        if layers is not None:
            self.layers = layers
        elif int4:
            # weights arrive quantised; the library expands them to the bf16 values the model computes with
            self.layers4 = [ks.make_int4_layer_on_device(s, l, "cuda") for l in range(s.n_layers)]
            self.layers = []
            for l in range(s.n_layers):
                wl = {n: kb.dequantize_int4(*self.layers4[l][n]) for n in ks.INT4_MATS}   # (codes, words, rows, K)
                wl["ln1"] = torch.ones(s.hidden, dtype=self.dt, device="cuda")
                wl["ln2"] = torch.ones(s.hidden, dtype=self.dt, device="cuda")
                wl["bq"] = wl["bk"] = wl["bv"] = None
                self.layers.append(wl)
        else:
            self.layers = [ks.make_layer_weights(s, l, "cuda") for l in range(s.n_layers)]
        self.embed = ks.make_embedding(s, "cuda")
        self.ids = ks.make_token_ids(self.n_tokens, s.vocab, 0)
        self.streams = [torch.cuda.Stream() for _ in range(3)]
        torch.cuda.synchronize()
        self.ctx = KeepContext(s, self.layers, self.embed, self.n_tokens + extra_tokens, self.G, kb.KEEP_KERNELS_AUTO,
                               *self.streams)
        if self.layers4 is not None:
            self.ctx.attach_int4(self.layers4)
        self.prompt = None
        self.random_cache = random_cache
        self.setup_s = time.perf_counter() - t0

    def make_prompt(self):
        """Group caches (outside every timed region) and the prompt that points at them."""
        from paper_2602_23592_amd import KeepPrompt
        torch, kb, w, s = self.torch, self.kb, self.w, self.s
        t0 = time.perf_counter()
        if self.random_cache:
            kb_all = torch.empty((s.n_layers, w.mem_tokens, s.n_kv_heads, s.head_dim), dtype=self.dt, device="cuda")
            vb_all = torch.empty_like(kb_all)
            gen = torch.Generator(device="cuda")
            gen.manual_seed(7)
            for l in range(s.n_layers):
                kb_all[l] = torch.randn(kb_all[l].shape, generator=gen, device="cuda").to(self.dt)
                vb_all[l] = torch.randn(vb_all[l].shape, generator=gen, device="cuda").to(self.dt)
        else:
            kb_all, vb_all = precompute_group_caches(self.ctx, w, self.glen, self.ids, torch)
        off = np.concatenate([[0], np.cumsum(self.glen)]).astype(np.int64)
        self.host = w.kv_location == "pinned_host"
        if self.host:
            kb_src = torch.empty(kb_all.shape, dtype=self.dt, pin_memory=True)
            vb_src = torch.empty(vb_all.shape, dtype=self.dt, pin_memory=True)
            kb_src.copy_(kb_all)
            vb_src.copy_(vb_all)
            del kb_all, vb_all
        else:
            kb_src, vb_src = kb_all, vb_all
        self.k_blocks = [[kb_src[l, off[g]:off[g + 1]] for g in range(self.G)] for l in range(s.n_layers)]
        self.v_blocks = [[vb_src[l, off[g]:off[g + 1]] for g in range(self.G)] for l in range(s.n_layers)]
        self.prompt = KeepPrompt(self.glen, self.lq, self.ids, self.k_blocks, self.v_blocks, s.n_layers,
                                 kb.KEEP_KV_PINNED_HOST if self.host else kb.KEEP_KV_DEVICE, self.kinds)
        self.k_cache = torch.empty((s.n_layers, self.n_tokens, s.n_kv_heads, s.head_dim), dtype=self.dt, device="cuda")
        self.v_cache = torch.empty_like(self.k_cache)
        self.x_final = torch.empty((self.lq, s.hidden), dtype=self.dt, device="cuda")
        torch.cuda.synchronize()
        self.setup_s += time.perf_counter() - t0

    def close(self):
        self.ctx.close()
        for n in ("k_blocks", "v_blocks", "prompt", "k_cache", "v_cache", "layers", "layers4", "embed", "ctx"):
            setattr(self, n, None)
        import gc
        gc.collect()
        self.torch.cuda.empty_cache()


def time_steps(fn, steps, warmup, torch):
    """Warm-up, then `steps` calls timed one by one between device synchronisations (host clock).
    Returns (list of ms, results of the calls)."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ms, res = [], []
    for _ in range(steps):
        t0 = time.perf_counter()
        res.append(fn())
        torch.cuda.synchronize()
        ms.append((time.perf_counter() - t0) * 1e3)
    return ms, res


def stats(ms):
    return {"ms_median": round(float(np.median(ms)), 3), "ms_min": round(float(np.min(ms)), 3),
            "ms_mean": round(float(np.mean(ms)), 3)}


def check_outputs(case, runs):
    """Sanity of what the timed steps produced: finite final rows and caches of the last step, nested sets,
    the same sets at every step (the run is deterministic)."""
    torch = case.torch
    assert bool(torch.isfinite(case.x_final.float()).all()), "non-finite value in x_final"
    assert bool(torch.isfinite(case.k_cache[-1].float()).all()) and bool(torch.isfinite(case.v_cache[-1].float()).all())
    sets0 = runs[0][0]
    for sets, _ in runs:
        assert sets == sets0, "the selected sets differ between steps"
    for a, b in zip(sets0, sets0[1:]):
        assert set(b) <= set(a), "sets are not nested"
    return True


def token_schedule(ks, w, L, sched):
    """Ratio schedule of the token-granularity scheme: as the workload's, with the first selection made from layer
    1's deviation (layer 0's is zero), so layers 0 and 1 recompute every token."""
    r = ks.ratio_schedule(w.ratio, L, sched)
    if L > 2:
        r[1] = 1.0
    return r


def extras(a, torch, ks, kb, main_case, main_ratios, sched):
    """Extra keys of the default line: the paper-literal count budget on the same prompt, the other workloads, and on
    the host-resident one the three loading modes and the token-granularity comparison (bytes loaded, TTFT)."""
    out = {}
    steps, warm = 3, 1
    c = main_case
    ms, runs = time_steps(lambda: c.ctx.prefill(c.prompt, main_ratios, c.w.hops, c.k_cache, c.v_cache, c.x_final,
                                                kb.KEEP_BUDGET_GROUP_COUNT, a.load_mode, want_report=True,
                                                gate_up_events_only=True), steps, warm, torch)
    rep = runs[-1][1]
    L = c.s.n_layers
    out["count_budget_reading"] = dict(stats(ms), tokens_per_s=round(c.n_tokens / (np.median(ms) * 1e-3), 1),
                                       rows_per_layer_mean=round(float(np.mean([rep.rows[l] for l in range(1, L)])), 1),
                                       set_sizes=[len(x) for x in runs[-1][0]],
                                       note="ratio %.2f counted in memories (ceil(r G) of the %d memories), the section's "
                                            "wording; the 16 long static groups fit such a budget" % (c.w.ratio, c.G))
    layers14 = c.layers
    c.ctx.close()
    for n in ("k_blocks", "v_blocks", "prompt", "k_cache", "v_cache"):
        setattr(c, n, None)
    torch.cuda.empty_cache()
    others = {}
    for name in ("qwen14b_64k_stress", "qwen7b_16k", "qwen32b_32k_host"):
        same_shape = ks.workload(name).shape == c.s
        oc = Case(name, a, torch, ks, kb, layers=layers14 if same_shape else None)
        if not same_shape:
            layers14 = None
            c.layers = None
            torch.cuda.empty_cache()
        oc.make_prompt()
        w = oc.w
        ratios = ks.ratio_schedule(w.ratio, w.shape.n_layers, w.schedule)
        mode = kb.KEEP_BUDGET_TOKENS if w.budget == "tokens" else kb.KEEP_BUDGET_GROUP_COUNT
        entry = {"tokens": oc.n_tokens, "groups": oc.G, "layers": w.shape.n_layers, "ratio": w.ratio, "hops": w.hops,
                 "kv": w.kv_location}
        modes = (("layer_balanced", 2),) if not oc.host else (("serial", 0), ("next_layer", 1), ("layer_balanced", 2))
        for mname, lm in modes:
            ms, runs = time_steps(lambda: oc.ctx.prefill(oc.prompt, ratios, w.hops, oc.k_cache, oc.v_cache, oc.x_final,
                                                         mode, lm, want_report=True, gate_up_events_only=True),
                                  steps, warm, torch)
            check_outputs(oc, runs)
            rep = runs[-1][1]
            e = dict(stats(ms), tokens_per_s=round(oc.n_tokens / (np.median(ms) * 1e-3), 1))
            if oc.host:
                e["bytes_loaded"] = int(sum(rep.bytes_loaded[l] for l in range(w.shape.n_layers)))
            entry[mname] = e
        if oc.host:
            # where loading, not compute, is the longer leg (half the recompute ratio): the loading modes again
            import dataclasses
            low = ks.ratio_schedule(w.ratio / 2, w.shape.n_layers, w.schedule)
            entry["ratio_%.2f" % (w.ratio / 2)] = {}
            for mname, lm in (("next_layer", 1), ("layer_balanced", 2)):
                ms, runs = time_steps(lambda: oc.ctx.prefill(oc.prompt, low, w.hops, oc.k_cache, oc.v_cache, oc.x_final,
                                                             mode, lm, want_report=True, gate_up_events_only=True),
                                      steps, warm, torch)
                rep = runs[-1][1]
                entry["ratio_%.2f" % (w.ratio / 2)][mname] = dict(
                    stats(ms), bytes_loaded=int(sum(rep.bytes_loaded[l] for l in range(w.shape.n_layers))))
            # the comparison the section draws: token granularity loads every block and updates in place
            tr = token_schedule(ks, w, w.shape.n_layers, w.schedule)
            ms, runs = time_steps(lambda: oc.ctx.prefill_tokens(oc.prompt, tr, oc.k_cache, oc.v_cache, oc.x_final,
                                                                load_mode=2, want_report=True), steps, warm, torch)
            rep = runs[-1][2]
            entry["token_granularity"] = dict(
                stats(ms), tokens_per_s=round(oc.n_tokens / (np.median(ms) * 1e-3), 1),
                bytes_loaded=int(sum(rep.bytes_loaded[l] for l in range(w.shape.n_layers))),
                rows_per_layer_mean=round(float(np.mean([rep.rows[l] for l in range(2, w.shape.n_layers)])), 1),
                note="same prompt and mean ratio; tokens chosen by K/V deviation from layer 1 on, every block of every "
                     "layer loaded, recomputed rows written in place")
        others[name] = entry
        oc.close()
    out["other_workloads"] = others
    return out


def sweep(a, torch, ks, kb):
    """BASELINE's stress sweep: recompute ratio 5/10/20/30 % x hops 1-4 on one prompt (default: the 65 536-token,
    1 024-memory one).  One JSON line per point."""
    c = Case(a.workload, a, torch, ks, kb)
    c.make_prompt()
    w, s, L = c.w, c.s, c.s.n_layers
    mode = kb.KEEP_BUDGET_TOKENS if (a.budget or w.budget) == "tokens" else kb.KEEP_BUDGET_GROUP_COUNT
    for ratio in (0.05, 0.10, 0.20, 0.30):
        ratios = ks.ratio_schedule(ratio, L, a.schedule or w.schedule)
        for hops in (1, 2, 3, 4):
            ms, runs = time_steps(lambda: c.ctx.prefill(c.prompt, ratios, hops, c.k_cache, c.v_cache, c.x_final, mode,
                                                        a.load_mode, want_report=True), a.steps, 1, torch)
            check_outputs(c, runs)
            rep = runs[-1][1]
            tot = lambda n: round(float(sum(getattr(rep, n)[l] for l in range(L))), 2)
            print(json.dumps(dict(stats(ms), workload=w.name, ratio=ratio, hops=hops,
                                  tokens_per_s=round(c.n_tokens / (np.median(ms) * 1e-3), 1),
                                  rows_per_layer_mean=round(float(np.mean([rep.rows[l] for l in range(1, L)])), 1),
                                  hops_run_layer0=int(rep.hops_run[0]), set_size_layer1=int(rep.set_size[1]),
                                  attn_rows_layer0=int(rep.attn_rows[0]),
                                  keys_per_attended_row=round(float(sum(rep.attn_keys[l] for l in range(L))) /
                                                              max(1.0, float(sum(rep.attn_rows[l] for l in range(L)))), 1),
                                  ms_gemms=round(tot("ms_qkv_gemm") + tot("ms_oproj") + tot("ms_gateup") + tot("ms_down"), 2),
                                  ms_attention=tot("ms_attn"), ms_score_select=tot("ms_score"),
                                  ms_realign=tot("ms_realign"), note="per-kernel sums from the fully instrumented steps "
                                  "(HIP events around every kernel add about 2 ms per step)")), flush=True)
    c.close()


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py measures one GPU: the selective-recompute prefill is built and measured on a single "
              "MI355X in this repository; run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import keep_synth as ks
    from paper_2602_23592_amd import KeepPrompt
    from paper_2602_23592_amd import binding as kb

    if not torch.cuda.is_available():
        print("bench.py needs a GPU (no CPU fallback exists)", file=sys.stderr)
        sys.exit(3)
    gate = ProfilerGate()
    gate.pause()                    # set-up (weights, group caches) is not part of the measurement
    if a.sweep:
        if a.workload == "qwen14b_32k":
            a.workload = "qwen14b_64k_stress"
        gate.resume()
        sweep(a, torch, ks, kb)
        return
    case = Case(a.workload, a, torch, ks, kb, ratio=a.ratio, sparse_rows=a.sparse_rows, int4=a.int4,
                random_cache=a.random_cache, extra_tokens=a.decode_tokens + 1)
    w, s, ctx = case.w, case.s, case.ctx
    sched = a.schedule or w.schedule
    budget = a.budget or w.budget
    budget_mode = kb.KEEP_BUDGET_TOKENS if budget == "tokens" else kb.KEEP_BUDGET_GROUP_COUNT
    glen, kinds, G, lq, n_tokens, dt, ids = case.glen, case.kinds, case.G, case.lq, case.n_tokens, case.dt, case.ids
    if a.memory_update:
        gate.resume()
        res = memory_update_cost(ctx, w, torch, a.steps, a.warmup)
        res["weights"] = "int4 weight-only (group 128) where a launch has at most 48 rows" if a.int4 else s.storage
        print(json.dumps(res))
        return
    case.make_prompt()
    prompt, host = case.prompt, case.host
    k_blocks, v_blocks = case.k_blocks, case.v_blocks
    k_cache, v_cache, x_final = case.k_cache, case.v_cache, case.x_final
    tokens_mode = a.granularity == "tokens"
    ratios = token_schedule(ks, w, s.n_layers, sched) if tokens_mode else ks.ratio_schedule(w.ratio, s.n_layers, sched)
    if a.sparse_rows > 0:
        ratios[:] = 0.0
    t_setup = case.setup_s

    def step(report, light=False):
        if tokens_mode:
            rows_t, _, rep_t = ctx.prefill_tokens(prompt, ratios, k_cache, v_cache, x_final, load_mode=a.load_mode,
                                                  want_report=report)
            return rows_t, rep_t
        return ctx.prefill(prompt, ratios, w.hops, k_cache, v_cache, x_final, budget_mode,
                           a.load_mode, want_report=report, gate_up_events_only=light)

    if a.decode_tokens > 0:
        gate.resume()
        print(json.dumps(decode_bench(ctx, prompt, ratios, w, s, n_tokens, budget_mode, a, torch, dt)))
        return

    gate.resume()
    if a.calib_copy_mib > 0:
        src = torch.empty(a.calib_copy_mib << 20, dtype=torch.uint8, device="cuda")
        src.zero_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(a.warmup):
        step(False)
    torch.cuda.synchronize()
    # Timed region: EXACTLY a.steps steps between two device synchronisations.  HIP events only around the roofline
    # kernel (the gate/up GEMM); a report with events around every kernel costs about 2 ms per step.  Each step is
    # also timed on its own (median / min); one more step with the full report follows, outside the timed region,
    # for the per-kernel table.
    light_reports, step_ms, runs = [], [], []
    t0 = time.perf_counter()
    for _ in range(a.steps):
        t1 = time.perf_counter()
        sets, rep = step(True, light=True)       # keep_prefill returns when its streams have drained
        step_ms.append((time.perf_counter() - t1) * 1e3)
        light_reports.append(rep)
        runs.append((sets, rep))
    torch.cuda.synchronize()
    dt_s = time.perf_counter() - t0
    ms_per_step = dt_s * 1e3 / max(1, a.steps)
    outputs_ok = check_outputs(case, runs)
    sets, full_rep = step(True)
    torch.cuda.synchronize()
    reports = [full_rep]
    gate.pause()

    # ---- per-kernel figures from the HIP-event report (averaged over the timed steps)
    L = s.n_layers
    rows = np.array([reports[-1].rows[l] for l in range(L)], dtype=np.float64)
    re_rows = np.array([reports[-1].realign_rows[l] for l in range(L)], dtype=np.float64)
    ffn_rows = np.array([reports[-1].ffn_rows[l] for l in range(L)], dtype=np.float64)
    # keys seen by the rows the attention actually ran on (at an evaluation-first layer only the rows whose
    # scores or outputs are read are attended)
    vis = np.array([reports[-1].attn_keys[l] for l in range(L)], dtype=np.float64)
    attn_rows = [int(reports[-1].attn_rows[l]) for l in range(L)]

    def mean_ms(name):
        return np.mean([[getattr(r, name)[l] for l in range(L)] for r in reports], axis=0)

    qd, kvd = s.n_q_heads * s.head_dim, s.n_kv_heads * s.head_dim
    esz = 2 if s.storage == "bf16" else 4
    kern = {}

    def add(name, ms, work, unit, peak):
        tot_ms = float(np.sum(ms))
        ach = float(np.sum(work)) / (tot_ms * 1e-3) if tot_ms > 0 else 0.0
        scale = 1e12 if unit == "TFLOP/s" else 1e9
        kern[name] = {"ms_per_step": round(tot_ms, 3), "achieved": round(ach / scale, 2), "unit": unit,
                      "frac": round(ach / scale / peak, 4)}

    add("gemm_gate_up_swiglu", mean_ms("ms_gateup"), 2.0 * ffn_rows * s.hidden * 2 * s.ffn_dim, "TFLOP/s", PEAK_BF16_TFLOPS)
    add("gemm_down", mean_ms("ms_down"), 2.0 * ffn_rows * s.hidden * s.ffn_dim, "TFLOP/s", PEAK_BF16_TFLOPS)
    add("gemm_qkv", mean_ms("ms_qkv_gemm"), 2.0 * rows * s.hidden * (qd + 2 * kvd), "TFLOP/s", PEAK_BF16_TFLOPS)
    add("gemm_out_proj", mean_ms("ms_oproj"), 2.0 * ffn_rows * qd * s.hidden, "TFLOP/s", PEAK_BF16_TFLOPS)
    if not tokens_mode:
        add("sparse_row_attention", mean_ms("ms_attn"), 4.0 * s.head_dim * s.n_q_heads * vis, "TFLOP/s", PEAK_BF16_TFLOPS)
    add("realign_concat", mean_ms("ms_realign"), 4.0 * re_rows * kvd * esz, "GB/s", PEAK_HBM_GBS)
    if float(np.sum(mean_ms("ms_rope"))) > 0.02 * L:
        add("rope_scatter", mean_ms("ms_rope"), rows * ((qd + 2 * kvd) * 4.0 + (qd + 3 * kvd) * esz), "GB/s", PEAK_HBM_GBS)
    else:   # bias, RoPE and the K/V scatter ran as the QKV projection's epilogue: no kernel of their own
        kern["rope_scatter"] = {"ms_per_step": 0.0, "fused_into": "gemm_qkv"}
    # score pass: Q.K^T of every recomputed row against the recomputed memory keys at or before it
    # (the same compact list), then the reductions and the selector; layers whose budget keeps all
    # or none of the candidates run no pass
    ms_sc = mean_ms("ms_score")
    mem = np.maximum(rows - lq, 0.0)
    pairs = np.where(ms_sc > 0, mem * (mem + 1) / 2 + lq * mem, 0.0)
    if not tokens_mode:
        add("score_select", ms_sc, 2.0 * s.head_dim * s.n_q_heads * pairs, "TFLOP/s", PEAK_BF16_TFLOPS)
    # attention in bytes too: one pass over the visible K and V per (row tile, KV head) is the algorithmic
    # minimum only when rows share tiles; report the cache-size figure (K_hat + V_hat of the layer, once)
    att_ms = float(np.sum(mean_ms("ms_attn")))
    if not tokens_mode:
        kern["sparse_row_attention"]["cache_gbs"] = round(L * 2.0 * n_tokens * kvd * esz / (att_ms * 1e-3) / 1e9, 1) if att_ms else 0

    # the roofline kernel from the timed steps themselves (the token-granularity run carries full reports)
    gu_ms = float(np.sum(np.mean([[r.ms_gateup[l] for l in range(L)] for r in light_reports], axis=0)))
    gu_work = float(np.sum(2.0 * ffn_rows * s.hidden * 2 * s.ffn_dim))
    gu = {"ms_per_step": round(gu_ms, 3), "achieved": round(gu_work / (gu_ms * 1e-3) / 1e12, 2),
          "frac": round(gu_work / (gu_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}
    kern["gemm_gate_up_swiglu"]["timed_region"] = gu
    n_launch = L
    # L2-miss bytes per launch: measured by rocprofv3 counter runs of this same command and stored under profiles/;
    # valid for the default workload and settings, and only while the kernel's source is the one that was measured
    default_run = (a.workload == "qwen14b_32k" and a.schedule is None and a.ratio is None and a.budget is None
                   and not a.random_cache and a.sparse_rows == 0 and not tokens_mode)
    traffic, traffic_src = stored_traffic() if default_run else (None, "not the workload of the stored counter run")
    roofline = {"kernel": "k_gemm_mfma<256,256,...,SWIGLU> + k_gemm_fixup (gate/up projection with fused SiLU*mul; "
                          "256x256 tiles, the last partly filled round cut along K)",
                "bound": "mfma", "achieved": gu["achieved"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": gu["frac"], "traffic": traffic, "traffic_source": traffic_src,
                "avg_launch_ms": round(gu["ms_per_step"] / n_launch, 4), "launches_per_step": n_launch}

    out = {
        "metric": "prefill tokens/s with KV reuse (TTFT in ms_per_step; sparse-attn HBM GB/s in sparse_attn_hbm)",
        "value": round(n_tokens / (ms_per_step * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(ms_per_step, 3),
        "ttft_ms": round(ms_per_step, 3), "ttft_ms_median": round(float(np.median(step_ms)), 3),
        "ttft_ms_min": round(float(np.min(step_ms)), 3), "outputs_checked": outputs_ok,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": s.storage, "data": "synthetic",
        "config": {"workload": "%s: %d layers, hidden %d, %d Q / %d KV heads, head_dim %d, FFN %d; %d tokens = %d "
                               "memory groups (%d tokens) + %d-token instruction; ratio %.2f of the %s (%s), %d hops; KV %s%s"
                               % (w.name, L, s.hidden, s.n_q_heads, s.n_kv_heads, s.head_dim, s.ffn_dim, n_tokens, G,
                                  w.mem_tokens, lq, w.ratio, budget, sched, w.hops, w.kv_location,
                                  "; TOKEN granularity (comparison scheme)" if tokens_mode else ""),
                   "rows_per_layer_mean": round(float(np.mean(rows[1:])) if L > 1 else float(rows[0]), 1),
                   "attn_rows_layer0": attn_rows[0], "rows_layer0": int(rows[0]), "ffn_rows_layer0": int(ffn_rows[0]), "set_sizes": [len(x) for x in sets],
                   "group_caches": "random draws" if a.random_cache else "library dense prefill of each group alone",
                   "load_mode": a.load_mode, "setup_s": round(t_setup, 1)},
        "roofline": roofline,
        "kernels": kern,
    }
    if host:
        out["bytes_loaded"] = int(sum(full_rep.bytes_loaded[l] for l in range(L)))
    if a.sparse_rows == 0 and not host and not tokens_mode:
        # the third figure of the metric: cache bytes per second of the sparse-row attention where it is bound by
        # reading the cache once (pure reuse, a 16-row instruction behind the same memories; outside the timed region)
        lq_s = 16
        n_s = w.mem_tokens + lq_s
        prompt_s = KeepPrompt(glen, lq_s, ids[:n_s], k_blocks, v_blocks, s.n_layers, kb.KEEP_KV_DEVICE, kinds)
        x_s = torch.empty((lq_s, s.hidden), dtype=dt, device="cuda")
        zeros = np.zeros(L, dtype=np.float32)
        reps_s = []
        for i in range(3):
            _, r_s = ctx.prefill(prompt_s, zeros, w.hops, k_cache, v_cache, x_s, budget_mode, a.load_mode,
                                 want_report=True, cache_rows=n_tokens)
            torch.cuda.synchronize()
            if i:
                reps_s.append(r_s)
        att_s = float(np.mean([sum(r.ms_attn[l] for l in range(L)) for r in reps_s]))
        gbs = L * 2.0 * n_s * kvd * esz / (att_s * 1e-3) / 1e9
        out["sparse_attn_hbm"] = {"rows": lq_s, "cache_tokens": n_s, "attn_ms_per_step": round(att_s, 3),
                                  "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                  "frac": round(gbs / PEAK_HBM_GBS, 4),
                                  "note": "K_hat + V_hat of every layer read once / time of the attention launches "
                                          "(work-list upload, kernel, combine of the key chunks)"}
    if a.layers_json:
        from paper_2602_23592_amd.binding import _REPORT_MS
        per_layer = {"rows": [int(v) for v in rows], "ffn_rows": [int(v) for v in ffn_rows],
                     "set_sizes": [len(x) for x in sets]}
        for name in _REPORT_MS:
            per_layer[name] = [round(float(v), 4) for v in mean_ms(name)]
        with open(a.layers_json, "w") as f:
            json.dump(per_layer, f)
    if default_run and not a.no_extras:
        out.update(extras(a, torch, ks, kb, case, ratios, sched))
    else:
        ctx.close()
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, glen, rows, n_tokens)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
