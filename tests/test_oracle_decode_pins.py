"""Pins of the oracle's first-token / greedy-decode functions (Section 1, Section 5)."""
import numpy as np
import torch
import torch.nn.functional as F

import keep_synth as ks
from oracle import keep_oracle as ko
from oracle_util import oracle_shape, small_problem, small_shape


def _head(shape, seed=5):
    rng = np.random.default_rng(seed)
    return 1.0 + 0.1 * rng.standard_normal(shape.hidden), 0.3 * rng.standard_normal((shape.vocab, shape.hidden))


def test_decoding_over_a_cache_equals_the_last_row_of_a_longer_dense_prefill():
    """The KV-cache identity: token n run alone over the cache of tokens 0..n-1 gives, at every layer,
    the K/V row and the hidden row that a dense causal prefill of tokens 0..n gives at row n."""
    shape = small_shape(n_q_heads=6, n_kv_heads=2, head_dim=8, hidden=48)
    sh, layers, embed, ids, _, _ = small_problem(shape, [13], 1)
    n = 13
    kf, vf, xf = ko.dense_prefill(sh, layers, embed, ids[:n + 1], 0)      # the longer sequence
    kp, vp, _ = ko.dense_prefill(sh, layers, embed, ids[:n], 0)           # the prompt alone
    kc = [np.concatenate([k, np.zeros((1,) + k.shape[1:])]) for k in kp]
    vc = [np.concatenate([v, np.zeros((1,) + v.shape[1:])]) for v in vp]
    x = embed[ids[n]].astype(np.float64)
    for l in range(sh.n_layers):
        x = ko.decode_layer(sh, layers[l], x, n, kc[l], vc[l])
        np.testing.assert_allclose(kc[l], kf[l], atol=1e-12)
        np.testing.assert_allclose(vc[l], vf[l], atol=1e-12)
    np.testing.assert_allclose(x, xf[n], atol=1e-11)


def test_greedy_decode_equals_repeated_dense_prefill():
    """Every greedy token equals the argmax at the last row of a dense prefill of prompt + tokens so far."""
    shape = small_shape(n_q_heads=4, n_kv_heads=2, head_dim=8, hidden=32)
    sh, layers, embed, ids, _, _ = small_problem(shape, [7], 1)
    fn, lm = _head(shape)
    n, n_new = 7, 4
    kp, vp, xp = ko.dense_prefill(sh, layers, embed, ids[:n], 0)
    pad = lambda c: [np.concatenate([t, np.zeros((n_new,) + t.shape[1:])]) for t in c]
    toks, logits = ko.greedy_decode(sh, layers, embed, fn, lm, xp[-1], pad(kp), pad(vp), n, n_new)
    seq = list(ids[:n])
    for t in range(n_new):
        _, _, xs = ko.dense_prefill(sh, layers, embed, np.asarray(seq), 0)
        ref = ko.lm_logits(sh, fn, lm, xs[-1:])[0]
        np.testing.assert_allclose(logits[t], ref, atol=1e-10)
        assert toks[t] == int(np.argmax(ref))
        seq.append(toks[t])


def test_logits_match_torch_expression():
    shape = small_shape(hidden=40)
    sh = oracle_shape(shape, "f64")
    fn, lm = _head(shape)
    x = np.random.default_rng(1).standard_normal((3, shape.hidden))
    got = ko.lm_logits(sh, fn, lm, x)
    xt = torch.from_numpy(x)
    ref = F.linear(F.rms_norm(xt, (shape.hidden,), torch.from_numpy(fn), sh.rms_eps), torch.from_numpy(lm)).numpy()
    np.testing.assert_allclose(got, ref, atol=1e-12)


def test_greedy_tie_takes_the_lowest_id_and_forcing_feeds_the_given_token():
    assert ko.greedy_token(np.array([0.5, 2.0, 2.0, -1.0, 2.0])) == 1
    shape = small_shape(n_q_heads=4, n_kv_heads=2, head_dim=8, hidden=32)
    sh, layers, embed, ids, _, _ = small_problem(shape, [5], 1)
    fn, lm = _head(shape)
    kp, vp, xp = ko.dense_prefill(sh, layers, embed, ids[:5], 0)
    pad = lambda c: [np.concatenate([t, np.zeros((2,) + t.shape[1:])]) for t in c]
    free, lg_free = ko.greedy_decode(sh, layers, embed, fn, lm, xp[-1], pad(kp), pad(vp), 5, 2)
    other = (free[0] + 1) % shape.vocab
    forced, lg_forced = ko.greedy_decode(sh, layers, embed, fn, lm, xp[-1], pad(kp), pad(vp), 5, 2, forced_tokens=[other])
    assert forced[0] == free[0]                                  # the reported choice is the free one
    np.testing.assert_allclose(lg_forced[0], lg_free[0], atol=0)
    _, _, xs = ko.dense_prefill(sh, layers, embed, np.asarray(list(ids[:5]) + [other]), 0)
    np.testing.assert_allclose(lg_forced[1], ko.lm_logits(sh, fn, lm, xs[-1:])[0], atol=1e-10)
