"""GPU parity of the first token and greedy decoding over the joined cache (Section 1, Section 5)
against the oracle, through the C ABI: logits of every step, the greedy choice, the appended K/V rows."""
import numpy as np
import pytest
import torch

import keep_synth as ks
from oracle import keep_oracle as ko
from gpu_util import Problem, max_rel, to_np
from paper_2602_23592_amd import KeepError

pytestmark = pytest.mark.gpu

F32 = ks.ModelShape(2, 128, 6, 2, 64, 200, 211, 1.0e6, 1e-6, "f32")
BF16 = ks.ModelShape(2, 512, 8, 2, 128, 1024, 1031, 1.0e6, 1e-6, "bf16")


def head_weights(shape, seed=17):
    g = torch.Generator().manual_seed(seed)
    dt = ks.torch_dtype(shape.storage)
    fn = (1.0 + 0.1 * torch.randn(shape.hidden, generator=g)).to(dt)
    lm = (0.05 * torch.randn(shape.vocab, shape.hidden, generator=g)).to(dt)
    return fn, lm


@pytest.mark.parametrize("shape,tol", [(F32, 1e-4), (BF16, 2e-2)], ids=["f32", "bf16_mfma"])
def test_prefill_then_decode_matches_oracle(shape, tol):
    glen, lq, n_new = [40, 7, 65, 30], 9, 5
    pb = Problem(shape, glen, lq, seed=6, std=0.05, bias=True)
    n = pb.n_tokens
    cap = n + n_new
    ctx, pr = pb.context(max_tokens=cap), pb.prompt()
    fn, lm = head_weights(shape)
    dt = ks.torch_dtype(shape.storage)
    L = shape.n_layers
    kc = torch.zeros((L, cap, shape.n_kv_heads, shape.head_dim), dtype=dt, device="cuda")
    vc = torch.zeros_like(kc)
    xf = torch.empty((lq, shape.hidden), dtype=dt, device="cuda")
    ratios = [1.0] + [0.5] * (L - 1)
    sets, _ = ctx.prefill(pr, ratios, 2, kc, vc, xf, cache_rows=cap)
    logits = torch.empty((n_new, shape.vocab), dtype=torch.float32, device="cuda")
    toks = ctx.decode(fn.cuda(), lm.cuda(), xf[-1], kc, vc, n, n_new, logits_out=logits)
    torch.cuda.synchronize()
    lg = to_np(logits)
    # the greedy choice is the argmax of the device's own logits (lowest id among equals): unique, bit-exact
    assert toks == [int(np.argmax(lg[t])) for t in range(n_new)]
    assert torch.all(kc[:, n + n_new - 1:] == 0) and torch.all(vc[:, n + n_new - 1:] == 0)   # nothing past the last fed token

    # oracle: same prefill (teacher-forced sets), then decoding fed with the device's tokens
    ref = ko.keep_prefill(pb.sh, pb.layers, pb.embed, pb.ids, glen, lq, pb.kb, pb.vb, ratios, 2, forced_sets=sets)
    pad = lambda c: [np.concatenate([t, np.zeros((n_new,) + t.shape[1:])]) for t in c]
    kr, vr = pad(ref["k_hat"]), pad(ref["v_hat"])
    rtoks, rlg = ko.greedy_decode(pb.sh, pb.layers, pb.embed, ks.to_numpy_f64(fn), ks.to_numpy_f64(lm), ref["x_final"][-1],
                                  kr, vr, n, n_new, forced_tokens=toks)
    for t in range(n_new):
        e = max_rel(lg[t], rlg[t])
        print(shape.storage, "step", t, "logits %.2e" % e, "token", toks[t], "oracle", rtoks[t])
        assert e < tol
        # the oracle's choice must be (nearly) as good under the device's logits: same decision up to the tolerance
        assert lg[t][rtoks[t]] >= lg[t].max() - 2 * tol * np.abs(rlg[t]).max()
    for l in range(L):
        assert max_rel(to_np(kc[l, :n + n_new - 1]), kr[l][:n + n_new - 1]) < tol
        assert max_rel(to_np(vc[l, :n + n_new - 1]), vr[l][:n + n_new - 1]) < tol


def test_decode_forced_tokens_and_single_token():
    shape = F32
    pb = Problem(shape, [12], 3, seed=8, std=0.1)
    n = pb.n_tokens
    ctx, pr = pb.context(max_tokens=n + 8), pb.prompt()
    fn, lm = head_weights(shape)
    kc = torch.zeros((2, n + 8, 2, 64), device="cuda")
    vc = torch.zeros_like(kc)
    xf = torch.empty((3, shape.hidden), device="cuda")
    ctx.prefill(pr, [1.0, 1.0], 1, kc, vc, xf, cache_rows=n + 8)
    first = ctx.decode(fn.cuda(), lm.cuda(), xf[-1], kc, vc, n, 1)          # first token only: no layer runs
    k_before = kc.clone()
    forced = [(first[0] + 5) % shape.vocab, 3]
    lg = torch.empty((3, shape.vocab), device="cuda")
    got = ctx.decode(fn.cuda(), lm.cuda(), xf[-1], kc, vc, n, 3, logits_out=lg, forced_tokens=forced)
    assert got[0] == first[0]
    assert torch.equal(kc[:, :n], k_before[:, :n])
    ref = ko.keep_prefill(pb.sh, pb.layers, pb.embed, pb.ids, [12], 3, pb.kb, pb.vb, [1.0, 1.0], 1)
    pad = lambda c: [np.concatenate([t, np.zeros((8,) + t.shape[1:])]) for t in c]
    _, rlg = ko.greedy_decode(pb.sh, pb.layers, pb.embed, ks.to_numpy_f64(fn), ks.to_numpy_f64(lm), ref["x_final"][-1],
                              pad(ref["k_hat"]), pad(ref["v_hat"]), n, 3, forced_tokens=forced)
    for t in range(3):
        assert max_rel(to_np(lg[t]), rlg[t]) < 1e-4


def test_decode_error_paths():
    shape = F32
    pb = Problem(shape, [4], 2, seed=1)
    ctx = pb.context(max_tokens=8)
    fn, lm = head_weights(shape)
    fn, lm = fn.cuda(), lm.cuda()
    kc = torch.zeros((2, 8, 2, 64), device="cuda")
    x = torch.zeros(shape.hidden, device="cuda")
    with pytest.raises(KeepError):
        ctx.decode(fn, lm, x, kc, kc.clone(), 6, 0)            # n_new out of range
    with pytest.raises(KeepError):
        ctx.decode(fn, lm, x, kc, kc.clone(), 6, 4)            # 6 + 4 - 1 > 8 rows
    with pytest.raises(KeepError):
        ctx.decode(fn, lm, x, kc, kc.clone(), 0, 1)            # empty context
    with pytest.raises(KeepError):
        ctx.decode(fn, lm, x, kc, kc.clone(), 4, 2, forced_tokens=[shape.vocab])
    xf = torch.empty((2, shape.hidden), device="cuda")
    with pytest.raises(KeepError):
        ctx.prefill(pb.prompt(), [1.0, 1.0], 1, kc, kc.clone(), xf, cache_rows=5)   # below the prompt's 6 tokens
