"""GPU parity of the INT4 weight-only path (Section 6.1: INT4 weight-only quantisation of the 32B model)
through the C ABI: the expansion to bfloat16 bit for bit, and the launches that read the 4-bit form
(a short prompt, the caching of one memory unit, greedy decoding) against the oracle run on the
dequantised weights."""
import numpy as np
import pytest
import torch

import keep_synth as ks
from oracle import int4_oracle as io
from oracle import keep_oracle as ko
from oracle_util import oracle_shape
from gpu_util import max_rel, to_np
from paper_2602_23592_amd import KeepContext, KeepError, KeepPrompt
from paper_2602_23592_amd.binding import dequantize_int4, KEEP_ERR_INVALID_ARG, KEEP_ERR_UNSUPPORTED, load_library

pytestmark = pytest.mark.gpu
TOL = 2e-2
SHAPE = ks.ModelShape(2, 512, 8, 2, 128, 1024, 1031, 1.0e6, 1e-6, "bf16")


def _dev(m):
    """storage arrays of a keep_synth INT4 matrix on the device, with its shape: (codes, words, rows, K)"""
    return (torch.from_numpy(m["codes"]).cuda(), torch.from_numpy(m["scale_zero"].view(np.int32)).cuda(),
            m["rows"], m["k"])


class Int4Problem:
    """Random INT4 layers: device tensors for the library, dequantised float64 matrices for the oracle."""

    def __init__(self, shape, std=0.05, seed=0):
        self.shape, self.sh = shape, oracle_shape(shape)
        g = torch.Generator().manual_seed(77 + seed)
        self.layers4_d, self.layers_d, self.layers = [], [], []
        for l in range(shape.n_layers):
            raw = ks.make_int4_layer(shape, l, std=std)
            dev4 = {n: _dev(raw[n]) for n in ks.INT4_MATS}
            wd = {n: dequantize_int4(*dev4[n]) for n in ks.INT4_MATS}            # the library's own expansion
            wo = {n: io.dequantize(raw[n]["codes"], raw[n]["scale_zero"], raw[n]["rows"], raw[n]["k"])
                  for n in ks.INT4_MATS}
            for n, width in (("ln1", shape.hidden), ("ln2", shape.hidden), ("bq", shape.q_dim), ("bk", shape.kv_dim),
                             ("bv", shape.kv_dim)):
                t = torch.randn(width, generator=g)
                t = (1.0 + 0.1 * t if n.startswith("ln") else std * t).to(torch.bfloat16)
                wd[n], wo[n] = t.cuda(), ks.to_numpy_f64(t)
            self.layers4_d.append(dev4); self.layers_d.append(wd); self.layers.append(wo)
        emb = torch.randn(shape.vocab, shape.hidden, generator=g).to(torch.bfloat16)
        self.embed_d, self.embed = emb.cuda(), ks.to_numpy_f64(emb)
        self.fn_t = (1.0 + 0.1 * torch.randn(shape.hidden, generator=g)).to(torch.bfloat16)
        self.lm_t = (0.05 * torch.randn(shape.vocab, shape.hidden, generator=g)).to(torch.bfloat16)

    def context(self, max_tokens, max_groups, int4=True):
        ctx = KeepContext(self.shape, self.layers_d, self.embed_d, max_tokens, max_groups)
        assert ctx.uses_mfma
        if int4:
            ctx.attach_int4(self.layers4_d)
        return ctx


@pytest.mark.parametrize("rows,k", [(32, 128), (224, 384), (512, 13824)])
def test_expansion_is_bit_exact(rows, k):
    m = ks.make_int4_matrix(rows, k, seed=rows + k, std=0.02)
    got = dequantize_int4(*_dev(m))
    torch.cuda.synchronize()
    want = torch.from_numpy(io.dequantize(m["codes"], m["scale_zero"], rows, k)).to(torch.bfloat16)   # exact: bf16 values
    assert torch.equal(got.cpu().view(torch.int16), want.view(torch.int16))


def test_expansion_covers_every_code_zero_pair_and_awkward_scales():
    """All 16 x 16 (code, zero) pairs under scales whose products need rounding to bfloat16."""
    rows, k = 16 * 4, 128
    q = np.tile(np.arange(16, dtype=np.uint8), (rows, k // 16))
    zero = np.repeat(np.arange(16, dtype=np.uint8), 4).reshape(rows, 1)
    scales = np.array([0.0131, 1.0 + 127.0 / 128, 3.3e-5, 7.77], dtype=np.float32)
    bits = np.tile(ks.bf16_bits_from_f32(scales), 16).reshape(rows, 1)
    codes, sz = ks.pack_int4_codes(q), ks.pack_int4_scale_zero(bits, zero)
    got = dequantize_int4(torch.from_numpy(codes).cuda(), torch.from_numpy(sz.view(np.int32)).cuda(), rows, k)
    want = torch.from_numpy(io.dequantize(codes, sz, rows, k)).to(torch.bfloat16)
    assert torch.equal(got.cpu().view(torch.int16), want.view(torch.int16))


def test_short_prompt_unit_caching_and_decode_read_the_int4_form():
    pb = Int4Problem(SHAPE)
    shape, sh, L = pb.shape, pb.sh, pb.shape.n_layers
    glen, lq, n_new = [36, 30], 9, 4
    n = sum(glen) + lq
    cap = n + n_new
    ids = ks.make_token_ids(n, shape.vocab, 3)
    ctx = pb.context(cap, len(glen))
    plain = pb.context(cap, len(glen), int4=False)

    # 1. caching memory units on their own: 36 rows (two row tiles per workgroup) and 30 rows (one)
    kb_d, vb_d = [[None] * len(glen) for _ in range(L)], [[None] * len(glen) for _ in range(L)]
    kb, vb = ko.precompute_group_caches(sh, pb.layers, pb.embed, ids, glen)
    off = 0
    for g, ln in enumerate(glen):
        k = torch.empty((L, ln, shape.n_kv_heads, shape.head_dim), dtype=torch.bfloat16, device="cuda")
        v = torch.empty_like(k)
        ctx.precompute_group(ids[off:off + ln], k, v)
        k2, v2 = torch.empty_like(k), torch.empty_like(v)
        plain.precompute_group(ids[off:off + ln], k2, v2)
        torch.cuda.synchronize()
        for l in range(L):
            assert max_rel(to_np(k[l]), kb[l][g]) < TOL and max_rel(to_np(v[l]), vb[l][g]) < TOL
            # same weights, another accumulation order: far inside the tolerance
            assert max_rel(to_np(k[l]), to_np(k2[l])) < TOL / 2 and max_rel(to_np(v[l]), to_np(v2[l])) < TOL / 2
            # the oracle's blocks (rounded to storage) feed both sides of the prefill below
            kb_d[l][g] = torch.from_numpy(kb[l][g]).to(torch.bfloat16).cuda()
            vb_d[l][g] = torch.from_numpy(vb[l][g]).to(torch.bfloat16).cuda()
            kb[l][g], vb[l][g] = to_np(kb_d[l][g]), to_np(vb_d[l][g])
        off += ln

    # 2. a prompt short enough that layer 1 (one memory of at most 36 rows + 9) runs on the weight-streaming kernels
    pr = KeepPrompt(glen, lq, ids, kb_d, vb_d, L)
    kc = torch.zeros((L, cap, shape.n_kv_heads, shape.head_dim), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    xf = torch.empty((lq, shape.hidden), dtype=torch.bfloat16, device="cuda")
    ratios = [1.0, 0.5]
    sets, rep = ctx.prefill(pr, ratios, 2, kc, vc, xf, cache_rows=cap, want_report=True)
    assert rep.rows[1] <= 48 < rep.rows[0]
    ref = ko.keep_prefill(sh, pb.layers, pb.embed, ids, glen, lq, kb, vb, ratios, 2, forced_sets=sets)
    for l in range(L):
        assert max_rel(to_np(kc[l, :n]), ref["k_hat"][l]) < TOL and max_rel(to_np(vc[l, :n]), ref["v_hat"][l]) < TOL
    assert max_rel(to_np(xf), ref["x_final"]) < TOL

    # 3. greedy decoding: every projection of every step reads the INT4 form (one row)
    logits = torch.empty((n_new, shape.vocab), dtype=torch.float32, device="cuda")
    toks = ctx.decode(pb.fn_t.cuda(), pb.lm_t.cuda(), xf[-1], kc, vc, n, n_new, logits_out=logits)
    torch.cuda.synchronize()
    pad = lambda c: [np.concatenate([t, np.zeros((n_new,) + t.shape[1:])]) for t in c]
    kr, vr = pad(ref["k_hat"]), pad(ref["v_hat"])
    rtoks, rlg = ko.greedy_decode(sh, pb.layers, pb.embed, ks.to_numpy_f64(pb.fn_t), ks.to_numpy_f64(pb.lm_t),
                                  ref["x_final"][-1], kr, vr, n, n_new, forced_tokens=toks)
    lg = to_np(logits)
    for t in range(n_new):
        e = max_rel(lg[t], rlg[t])
        print("int4 decode step", t, "logits %.2e" % e)
        assert e < TOL
        assert toks[t] == int(np.argmax(lg[t]))
    for l in range(L):
        assert max_rel(to_np(kc[l, :n + n_new - 1]), kr[l][:n + n_new - 1]) < TOL
        assert max_rel(to_np(vc[l, :n + n_new - 1]), vr[l][:n + n_new - 1]) < TOL
    # detaching returns to the bfloat16 launches
    ctx.attach_int4(None)
    lg2 = torch.empty_like(logits)
    kc2, vc2 = kc.clone(), vc.clone()
    ctx.decode(pb.fn_t.cuda(), pb.lm_t.cuda(), xf[-1], kc2, vc2, n, n_new, logits_out=lg2, forced_tokens=toks[:-1])
    assert max_rel(to_np(lg2), lg) < TOL / 2


def test_int4_error_paths():
    lib = load_library()
    m = ks.make_int4_matrix(32, 128, seed=1)
    codes, sz, _, _ = _dev(m)
    out = torch.empty((32, 128), dtype=torch.bfloat16, device="cuda")
    assert lib.keep_dequantize_int4(codes.data_ptr(), sz.data_ptr(), 32, 100, out.data_ptr(), None) == KEEP_ERR_INVALID_ARG
    assert lib.keep_dequantize_int4(None, sz.data_ptr(), 32, 128, out.data_ptr(), None) == KEEP_ERR_INVALID_ARG
    assert lib.keep_dequantize_int4(codes.data_ptr(), sz.data_ptr(), 0, 128, out.data_ptr(), None) == KEEP_ERR_INVALID_ARG
    assert lib.keep_dequantize_int4(codes.data_ptr(), sz.data_ptr(), 33, 128, out.data_ptr(), None) == KEEP_ERR_INVALID_ARG
    assert b"128" in lib.keep_last_error(None)
    # a context on the generic fp32 path has no INT4 launches
    f32 = ks.ModelShape(1, 128, 2, 1, 64, 256, 50, 1.0e6, 1e-6, "f32")
    layers, embed = ks.make_weights(f32, "cuda")
    ctx = KeepContext(f32, layers, embed, 16, 1)
    raw = ks.make_int4_layer(f32, 0)
    with pytest.raises(KeepError) as e:
        ctx.attach_int4([{n: _dev(raw[n]) for n in ks.INT4_MATS}])
    assert e.value.status == KEEP_ERR_UNSUPPORTED
    # a NULL pointer inside
    pb = Int4Problem(ks.ModelShape(1, 256, 2, 1, 128, 256, 50, 1.0e6, 1e-6, "bf16"))
    ctx = pb.context(16, 1, int4=False)
    from paper_2602_23592_amd.binding import LayerWeightsInt4
    arr = (LayerWeightsInt4 * 1)()
    assert ctx.lib.keep_attach_int4(ctx.handle, arr) == KEEP_ERR_INVALID_ARG


@pytest.mark.parametrize("workload", ["qwen14b_32k", "qwen32b_32k_host"])
def test_fullsize_projections_read_the_int4_form(workload):
    """One layer of the Qwen-14B shape (K = 5120 and 13 824, N up to 27 648) and of the Qwen-32B shape, the one the
    paper runs with INT4 weights (Section 6.1; FFN 27 648: K up to 27 648, N up to 55 296): a 48-token unit cached on its own
    (two row tiles per workgroup) and one decoded token (one row) with the 4-bit form attached, against the
    oracle on the dequantised weights.  Codes are uniform draws here (the binomial recipe takes minutes at
    this size on the host)."""
    full = ks.workload(workload).shape
    shape = ks.ModelShape(1, full.hidden, full.n_q_heads, full.n_kv_heads, full.head_dim, full.ffn_dim, 1031,
                          full.rope_theta, full.rms_eps, "bf16")
    sh = oracle_shape(shape)
    dev4 = ks.make_int4_layer_on_device(shape, 0, "cuda", std=0.02)
    wd = {n: dequantize_int4(*dev4[n]) for n in ks.INT4_MATS}
    wo = {n: io.dequantize(dev4[n][0].cpu().numpy(), dev4[n][1].cpu().numpy().view(np.uint32), dev4[n][2], dev4[n][3])
          for n in ks.INT4_MATS}
    for n in ks.INT4_MATS:   # the library's expansion is the oracle's, bit for bit, at full size too
        assert torch.equal(wd[n].cpu().view(torch.int16), torch.from_numpy(wo[n]).to(torch.bfloat16).view(torch.int16)), n
    g = torch.Generator().manual_seed(5)
    for n in ("ln1", "ln2"):
        t = (1.0 + 0.1 * torch.randn(shape.hidden, generator=g)).to(torch.bfloat16)
        wd[n], wo[n] = t.cuda(), ks.to_numpy_f64(t)
    wd["bq"] = wd["bk"] = wd["bv"] = None
    wo["bq"] = wo["bk"] = wo["bv"] = None
    emb = torch.randn(shape.vocab, shape.hidden, generator=g).to(torch.bfloat16)
    fn = torch.ones(shape.hidden, dtype=torch.bfloat16)
    lm = (0.05 * torch.randn(shape.vocab, shape.hidden, generator=g)).to(torch.bfloat16)
    n_unit, cap = 48, 52
    ctx = KeepContext(shape, [wd], emb.cuda(), cap, 1)
    assert ctx.uses_mfma
    ctx.attach_int4([dev4])
    ids = ks.make_token_ids(n_unit, shape.vocab, 9)
    kc = torch.zeros((1, cap, shape.n_kv_heads, shape.head_dim), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    k = torch.empty((1, n_unit, shape.n_kv_heads, shape.head_dim), dtype=torch.bfloat16, device="cuda")
    v = torch.empty_like(k)
    ctx.precompute_group(ids, k, v)
    kb, vb = ko.precompute_group_caches(sh, [wo], ks.to_numpy_f64(emb), ids, [n_unit])
    assert max_rel(to_np(k[0]), kb[0][0]) < TOL and max_rel(to_np(v[0]), vb[0][0]) < TOL
    # one decoded token over that unit as the context (K/V of the unit from the oracle, rounded to storage)
    kc[0, :n_unit] = torch.from_numpy(kb[0][0]).to(torch.bfloat16).cuda()
    vc[0, :n_unit] = torch.from_numpy(vb[0][0]).to(torch.bfloat16).cuda()
    x_last = (0.5 * torch.randn(shape.hidden, generator=g)).to(torch.bfloat16)
    logits = torch.empty((2, shape.vocab), dtype=torch.float32, device="cuda")
    toks = ctx.decode(fn.cuda(), lm.cuda(), x_last.cuda(), kc, vc, n_unit, 2, logits_out=logits)
    torch.cuda.synchronize()
    kr = [np.concatenate([to_np(kc[0, :n_unit]), np.zeros((cap - n_unit,) + kb[0][0].shape[1:])])]
    vr = [np.concatenate([to_np(vc[0, :n_unit]), np.zeros((cap - n_unit,) + vb[0][0].shape[1:])])]
    _, rlg = ko.greedy_decode(sh, [wo], ks.to_numpy_f64(emb), ks.to_numpy_f64(fn), ks.to_numpy_f64(lm),
                              ks.to_numpy_f64(x_last), kr, vr, n_unit, 2, forced_tokens=toks)
    lg = to_np(logits)
    for t in range(2):
        e = max_rel(lg[t], rlg[t])
        print("full-size int4 decode step", t, "logits %.2e" % e)
        assert e < TOL
    assert max_rel(to_np(kc[0, n_unit]), kr[0][n_unit]) < TOL and max_rel(to_np(vc[0, n_unit]), vr[0][n_unit]) < TOL
