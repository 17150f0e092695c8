"""CPU oracle for KEEP's selective KV recomputation (TEST INFRASTRUCTURE).

This file is test infrastructure, not product code.  Only the test-suite, the
smoke check and the bench's `cpu_baseline` leg may import it; the HIP library
and its Python binding never do, and it imports nothing from them.

It is a plain, slow numpy implementation (float64 arithmetic by default) of
what the hot path computes, step by step in the order the paper gives:

  * memory groups whose KV caches were computed independently are joined into
    one prompt, instruction last                       (Section 1; Section 4.1)
  * layer 0 recomputes every memory, later layers only the memories in the
    relevant set found at the previous layer           (Section 4.2, last par.)
  * per layer (`prefill_layer`, Section 5): QKV of the recomputed tokens,
    their causal attention over the whole joined cache, refreshed K/V written
    back, then output projection and FFN
  * importance evaluation (Section 4.2, the four bullet steps; Section 5
    `importance_evaluation`): initialisation from the query's average
    attention, top-ratio relevant set, propagation from the relevant set,
    convergence check
  * a memory not recomputed at one layer is never recomputed later
    (Section 4.3, the key observation), so relevant sets are nested.

The paper is KEEP's prose only: it prints no formula for the scores.  Each
choice below that the text leaves open is marked "reading:" and is listed in
the design notes of the repository.

Pins (tests under tests/, marker "not gpu"): dense layer vs an independent
PyTorch-CPU expression; ratio 1 == dense causal prefill; ratio 0 == re-rotated
concatenation; lone group reproduces its cache; RoPE composition and the
relative-position property; first-group and layer-0 invariances; attention-mass
conservation; harmonic closed form under uniform attention; brute-force top-k
and token-budget walks; hand-built propagation chains; decoding one token over
a cache == the last row of a dense prefill of the longer sequence; logits vs an
independent PyTorch-CPU expression; argmax tie rule; token-granularity variant:
ratio 1 == dense prefill, whole memories forced == the memory-granularity path,
zero deviation at layer 0 and for the first memory, top-k by brute force.
Parity unpinned: whether the selected memories are the ones a trained model
needs (task success rate) -- that needs the paper's datasets and weights.
"""
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

BUDGET_GROUP_COUNT = 0
BUDGET_TOKENS = 1

# Slack (in units of groups, or of tokens) that absorbs the binary32 rounding of a
# ratio before the ceiling / floor that turns it into a count.
BUDGET_EPS = 1.0e-3


@dataclass
class Shape:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn_dim: int
    vocab: int
    rope_theta: float = 1.0e6
    rms_eps: float = 1.0e-6
    storage: str = "f32"      # format in which K/V caches are stored: "f32", "bf16" or "f64" (no rounding)


# ----------------------------------------------------------------------------
# storage rounding
# ----------------------------------------------------------------------------
def round_to_storage(x: np.ndarray, storage: str) -> np.ndarray:
    """Value of `x` after being written to the cache format and read back."""
    if storage == "f64":
        return np.asarray(x)
    x32 = np.asarray(x).astype(np.float32)
    if storage == "f32":
        return x32.astype(x.dtype)
    if storage == "bf16":
        u = x32.view(np.uint32)
        keep = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
        return keep.view(np.float32).astype(x.dtype)
    raise ValueError(storage)


# ----------------------------------------------------------------------------
# rotary position embedding, rotate-half pairing (reading: the Qwen-2.5
# convention, since the paper's models are Qwen-2.5, Section 6.1)
# ----------------------------------------------------------------------------
def rope_cos_sin(positions: np.ndarray, head_dim: int, theta: float) -> Tuple[np.ndarray, np.ndarray]:
    """cos and sin of position * theta^(-2j/head_dim), j < head_dim/2, in float64."""
    j = np.arange(head_dim // 2, dtype=np.float64)
    freq = np.power(float(theta), -2.0 * j / head_dim)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * freq[None, :]
    return np.cos(ang), np.sin(ang)


def rotate(x: np.ndarray, positions: np.ndarray, theta: float) -> np.ndarray:
    """Rot(p) applied to every head vector of x[rows, heads, head_dim]."""
    dh = x.shape[-1]
    half = dh // 2
    c, s = rope_cos_sin(positions, dh, theta)
    c = c[:, None, :].astype(x.dtype)
    s = s[:, None, :].astype(x.dtype)
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


# ----------------------------------------------------------------------------
# building blocks of a pre-norm decoder layer
# ----------------------------------------------------------------------------
def rmsnorm(x: np.ndarray, w: np.ndarray, eps: float) -> np.ndarray:
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * w


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def _linear(x: np.ndarray, w: np.ndarray, b: Optional[np.ndarray]) -> np.ndarray:
    y = x @ w.T
    return y if b is None else y + b


def project_qkv(sh: Shape, w: Dict[str, np.ndarray], x: np.ndarray, positions: np.ndarray):
    """RMSNorm, Q/K/V projections and RoPE at the rows' global positions."""
    h = rmsnorm(x, w["ln1"], sh.rms_eps)
    n = x.shape[0]
    q = _linear(h, w["wq"], w.get("bq")).reshape(n, sh.n_q_heads, sh.head_dim)
    k = _linear(h, w["wk"], w.get("bk")).reshape(n, sh.n_kv_heads, sh.head_dim)
    v = _linear(h, w["wv"], w.get("bv")).reshape(n, sh.n_kv_heads, sh.head_dim)
    return rotate(q, positions, sh.rope_theta), rotate(k, positions, sh.rope_theta), v


def output_and_ffn(sh: Shape, w: Dict[str, np.ndarray], x: np.ndarray, attn_out: np.ndarray) -> np.ndarray:
    """Output projection, residual, RMSNorm, SwiGLU FFN, residual."""
    n = x.shape[0]
    x = x + attn_out.reshape(n, sh.n_q_heads * sh.head_dim) @ w["wo"].T
    h2 = rmsnorm(x, w["ln2"], sh.rms_eps)
    return x + (silu(h2 @ w["wgate"].T) * (h2 @ w["wup"].T)) @ w["wdown"].T


# ----------------------------------------------------------------------------
# textbook dense causal layer / prefill (used to precompute group caches and
# as the fixed point the selective path must reach at ratio 1)
# ----------------------------------------------------------------------------
def dense_layer(sh: Shape, w: Dict[str, np.ndarray], x: np.ndarray, positions: np.ndarray):
    """One decoder layer over a whole sequence with a lower-triangular mask.

    Returns (x_out, K, V) with K, V rounded to the cache format and attention
    computed from the rounded values (the cache is what attention reads).
    """
    n = x.shape[0]
    q, k, v = project_qkv(sh, w, x, positions)
    k = round_to_storage(k, sh.storage)
    v = round_to_storage(v, sh.storage)
    rep = sh.n_q_heads // sh.n_kv_heads
    allowed = np.tril(np.ones((n, n), dtype=bool))
    o = np.empty_like(q)
    for h in range(sh.n_q_heads):
        s = (q[:, h, :] @ k[:, h // rep, :].T) / np.sqrt(float(sh.head_dim))
        s = np.where(allowed, s, -np.inf)
        p = np.exp(s - s.max(axis=1, keepdims=True))
        p = p / p.sum(axis=1, keepdims=True)
        o[:, h, :] = p @ v[:, h // rep, :]
    return output_and_ffn(sh, w, x, o), k, v


def dense_prefill(sh: Shape, layers: Sequence[Dict[str, np.ndarray]], embed: np.ndarray,
                  token_ids: np.ndarray, first_position: int = 0, dtype=np.float64):
    """Dense causal prefill of `token_ids` placed at positions first_position, +1, ...

    Returns (K[l], V[l] lists of [n, n_kv_heads, head_dim], x_final [n, hidden])."""
    n = len(token_ids)
    positions = np.arange(first_position, first_position + n)
    x = embed[np.asarray(token_ids)].astype(dtype)
    ks, vs = [], []
    for l in range(sh.n_layers):
        x, k, v = dense_layer(sh, layers[l], x, positions)
        ks.append(k)
        vs.append(v)
    return ks, vs, x


def precompute_group_caches(sh: Shape, layers, embed, token_ids: np.ndarray, group_len: Sequence[int],
                            dtype=np.float64):
    """KV caches of each memory group computed on its own, at group-local
    positions 0..len-1 with attention inside the group only (Section 4.1: a static
    group is one jointly computed unit, a dynamic segment is its own unit).

    Returns k_blocks[l][g], v_blocks[l][g], each [len_g, n_kv_heads, head_dim]."""
    k_blocks = [[] for _ in range(sh.n_layers)]
    v_blocks = [[] for _ in range(sh.n_layers)]
    off = 0
    for n in group_len:
        ks, vs, _ = dense_prefill(sh, layers, embed, token_ids[off:off + n], 0, dtype)
        for l in range(sh.n_layers):
            k_blocks[l].append(ks[l])
            v_blocks[l].append(vs[l])
        off += n
    return k_blocks, v_blocks


# ----------------------------------------------------------------------------
# joining the caches: offsets, position re-alignment, concatenation
# ----------------------------------------------------------------------------
def group_offsets(group_len: Sequence[int]) -> np.ndarray:
    off = np.zeros(len(group_len) + 1, dtype=np.int64)
    off[1:] = np.cumsum(np.asarray(group_len, dtype=np.int64))
    return off


def realign_concat(sh: Shape, k_blocks_l: Sequence[np.ndarray], v_blocks_l: Sequence[np.ndarray],
                   group_len: Sequence[int], instr_len: int, dtype=np.float64):
    """Joined cache of one layer, [N, n_kv_heads, head_dim]: group g's keys, cached
    rotated at local positions j, are rotated on by the group's start offset so that
    they sit at global position off_g + j (rotations compose additively); values are
    copied.  Instruction rows are left zero: they are always computed.
    Reading: the paper never mentions positions; this is what independent per-group
    caching (Section 4.1) needs for the joined prompt to mean what it says."""
    off = group_offsets(group_len)
    n_total = int(off[-1]) + instr_len
    k_hat = np.zeros((n_total, sh.n_kv_heads, sh.head_dim), dtype=dtype)
    v_hat = np.zeros_like(k_hat)
    for g, n in enumerate(group_len):
        shift = np.full(n, off[g], dtype=np.int64)
        k_hat[off[g]:off[g] + n] = round_to_storage(rotate(k_blocks_l[g].astype(dtype), shift, sh.rope_theta),
                                                    sh.storage)
        v_hat[off[g]:off[g] + n] = v_blocks_l[g]
    return k_hat, v_hat


def rows_of(groups: Sequence[int], group_len: Sequence[int], instr_len: int) -> np.ndarray:
    """Global positions of the recomputed tokens: the groups' tokens in prompt
    order, then every instruction token (reading: the instruction has no cache, so
    it is computed at every layer)."""
    off = group_offsets(group_len)
    parts = [np.arange(off[g], off[g + 1]) for g in sorted(groups)]
    parts.append(np.arange(off[-1], off[-1] + instr_len))
    return np.concatenate(parts).astype(np.int64)


# ----------------------------------------------------------------------------
# one selective layer (`prefill_layer`, Section 5) with its attention scores
# ----------------------------------------------------------------------------
def selective_layer(sh: Shape, w: Dict[str, np.ndarray], x: np.ndarray, groups: Sequence[int],
                    group_len: Sequence[int], instr_len: int, k_hat: np.ndarray, v_hat: np.ndarray,
                    want_scores: bool = True, only_rows: Optional[np.ndarray] = None,
                    score_blocks: Optional[Sequence[int]] = None, probe: Optional[dict] = None):
    """Recompute the KV of the memories in `groups` (and of the instruction) over the
    joined cache of this layer.

    x[n_l, hidden] holds the hidden rows of the recomputed tokens in prompt order.
    k_hat / v_hat are updated in place at those tokens' positions.

    Returns (x_out[n_l, hidden], lse[n_l, n_q_heads], S) where S is the
    (len(groups)+1) x len(groups) group-score matrix (last row: the query), or None.

    only_rows: optional indices into the n_l rows; when given, attention and
    everything after it is evaluated for just those rows (K/V are still refreshed
    for all rows, since every later row attends to them) and x_out has that many
    rows.  S is then not available.

    score_blocks: optional list of source blocks (indices into `groups`, or
    len(groups) for the query); attention is then evaluated for all rows of just
    those blocks and S comes back with only those rows filled (NaN elsewhere);
    x_out and lse hold those blocks' rows in order.  For sampled checks at sizes
    where the full matrix is too slow.

    probe: optional dict that receives intermediate values for tests: "attn_out"
    [rows, n_q_heads, head_dim], the attention output of the evaluated rows before
    the output projection.
    """
    groups = sorted(int(g) for g in groups)
    assert instr_len >= 1 and min(group_len) >= 1      # a query is needed; blocks are non-empty
    off = group_offsets(group_len)
    n_total = k_hat.shape[0]
    pos = rows_of(groups, group_len, instr_len)
    assert x.shape[0] == len(pos)
    q, k, v = project_qkv(sh, w, x, pos)
    # refreshed K/V go into the cache (in its storage format) before attention reads it
    k_hat[pos] = round_to_storage(k, sh.storage)
    v_hat[pos] = round_to_storage(v, sh.storage)

    m = len(groups)
    block_starts = np.zeros(m + 2, dtype=np.int64)
    block_starts[1:m + 1] = np.cumsum([group_len[g] for g in groups])
    block_starts[m + 1] = block_starts[m] + instr_len
    if score_blocks is not None:
        assert only_rows is None and want_scores
        score_blocks = sorted(int(b) for b in score_blocks)
        only = np.concatenate([np.arange(block_starts[b], block_starts[b + 1]) for b in score_blocks])
        q, pos_q, x_res = q[only], pos[only], x[only]
    elif only_rows is not None:
        assert not want_scores
        q, pos_q, x_res = q[only_rows], pos[only_rows], x[only_rows]
    else:
        pos_q, x_res = pos, x
    n = len(pos_q)
    rep = sh.n_q_heads // sh.n_kv_heads
    visible = np.arange(n_total)[None, :] <= pos_q[:, None]        # key j is seen by row t iff j <= p_t
    o = np.empty_like(q)
    lse = np.empty((n, sh.n_q_heads), dtype=q.dtype)

    # partition of the evaluated rows and of the N keys into blocks, for the score sums
    if want_scores:
        if score_blocks is None:
            row_starts = block_starts[:m + 1]                           # block m = instruction rows
            n_row_blocks = m + 1
        else:
            lens = [block_starts[b + 1] - block_starts[b] for b in score_blocks]
            row_starts = np.concatenate([[0], np.cumsum(lens)[:-1]]).astype(np.int64)
            n_row_blocks = len(score_blocks)
        key_starts = off.copy()                                         # G group blocks, block G = instruction
        mass = np.zeros((n_row_blocks, len(group_len) + 1), dtype=q.dtype)

    for h in range(sh.n_q_heads):
        s = (q[:, h, :] @ k_hat[:, h // rep, :].T) / np.sqrt(float(sh.head_dim))
        s = np.where(visible, s, -np.inf)
        smax = s.max(axis=1, keepdims=True)
        e = np.exp(s - smax)
        denom = e.sum(axis=1, keepdims=True)
        p = e / denom
        lse[:, h] = (smax + np.log(denom))[:, 0]
        o[:, h, :] = p @ v_hat[:, h // rep, :]
        if want_scores:
            # attention mass sent by each row block to each key block, summed over heads
            by_key = np.add.reduceat(p, key_starts, axis=1)          # [n_l, G+1]
            mass += np.add.reduceat(by_key, row_starts, axis=0)      # [m+1, G+1]

    if probe is not None:
        probe["attn_out"] = o
    x_out = output_and_ffn(sh, w, x_res, o)
    scores = None
    if want_scores and score_blocks is None:
        scores = scores_from_mass(mass, groups, group_len, instr_len, sh.n_q_heads)
    elif want_scores:
        full = np.zeros((m + 1, len(group_len) + 1), dtype=mass.dtype)
        full[score_blocks] = mass
        scores = scores_from_mass(full, groups, group_len, instr_len, sh.n_q_heads)
        missing = [b for b in range(m + 1) if b not in score_blocks]
        scores[missing] = np.nan
    return x_out, lse, scores


def scores_from_mass(mass: np.ndarray, groups: Sequence[int], group_len: Sequence[int], instr_len: int,
                     n_q_heads: int) -> np.ndarray:
    """Average attention between memories (Section 4.2, initialisation and propagation
    steps): S[a, b] = attention mass from the rows of a to the keys of b, divided by
    heads x rows x keys.  Source rows: the candidate memories then the query (last
    row); target columns: the candidate memories.
    Reading: "average" is per head, per source row and per target key, so that long
    memories are not favoured; a memory's attention to itself is set to zero (it is
    in every cache already); attention to later memories is zero by causality.
    `mass` is [(m+1), G+1] over all key blocks (instruction last)."""
    m = len(groups)
    s = np.zeros((m + 1, m), dtype=mass.dtype)
    for i, a in enumerate(list(groups) + [None]):
        len_a = instr_len if a is None else group_len[a]
        if len_a == 0:
            continue
        for j, b in enumerate(groups):
            if a is not None and a == b:
                continue
            s[i, j] = mass[i, b] / (n_q_heads * float(len_a) * float(group_len[b]))
    return s


# ----------------------------------------------------------------------------
# multi-hop importance propagation and selection (`importance_evaluation`)
# ----------------------------------------------------------------------------
def budget_count(ratio: float, n_groups_total: int, n_candidates: int) -> int:
    """Number of memories to keep: ratio of the prompt's memories, rounded up
    (reading: the share r_i of Section 4.2 is a share of the memories of the whole prompt)."""
    k = int(np.ceil(float(np.float32(ratio)) * n_groups_total - BUDGET_EPS))
    return max(0, min(n_candidates, k))


def budget_tokens(ratio: float, mem_tokens: int) -> int:
    return int(np.floor(float(np.float32(ratio)) * mem_tokens + BUDGET_EPS))


def _ranked(importance: np.ndarray) -> List[int]:
    """Candidate indices by importance descending, index ascending on ties."""
    return sorted(range(len(importance)), key=lambda b: (-float(importance[b]), b))


def _take(importance: np.ndarray, mode: int, k: int, token_budget: int, cand_len: Sequence[int]) -> List[int]:
    order = _ranked(importance)
    if mode == BUDGET_GROUP_COUNT:
        return sorted(order[:k])
    used, out = 0, []
    for b in order:
        if used + cand_len[b] <= token_budget:
            out.append(b)
            used += cand_len[b]
    return sorted(out)


def select_multihop(S: np.ndarray, groups: Sequence[int], group_len: Sequence[int], ratio_next: float,
                    hops: int, mode: int = BUDGET_GROUP_COUNT, drop_query: bool = False):
    """Relevant set for the next layer from the score matrix S[(m+1), m] of this layer.

    All arithmetic is binary32 in a fixed order (sums over candidates in ascending
    order), because these floating-point values decide integers and the GPU selector
    must reach the same ones from the same S.

    Steps (Section 4.2): row-normalise S over the candidate targets (reading of the
    normalised scores that Fig. 6 shows: each source spreads one unit);
    initial importance = the query's row; relevant set = top of the importance order
    within the budget; new importance = average of the normalised rows of the query
    and of the relevant memories (reading: the query stays a source; `drop_query`
    gives the literal variant that averages over the relevant memories alone);
    stop when the set repeats or after `hops` selections.

    Returns (sorted next groups, number of selections run).
    """
    groups = [int(g) for g in groups]
    m = len(groups)
    assert S.shape == (m + 1, m)
    n_groups_total = len(group_len)
    mem_tokens = int(np.sum(group_len))
    cand_len = [int(group_len[g]) for g in groups]
    k = budget_count(ratio_next, n_groups_total, m)
    tok = budget_tokens(ratio_next, mem_tokens)
    if m == 0:
        return [], 0
    if mode == BUDGET_GROUP_COUNT:
        if k >= m:
            return list(groups), 0
        if k == 0:
            return [], 0
    else:
        if tok >= sum(cand_len):
            return list(groups), 0
        if tok <= 0:
            return [], 0

    s32 = np.asarray(S, dtype=np.float32)
    norm = np.zeros_like(s32)
    for a in range(m + 1):
        total = np.float32(0.0)
        for b in range(m):
            total = np.float32(total + s32[a, b])
        if total > 0:
            norm[a, :] = s32[a, :] / total
    importance = norm[m, :].copy()
    rel = _take(importance, mode, k, tok, cand_len)
    runs = 1
    while runs < max(1, hops):
        if drop_query:
            acc = np.zeros(m, dtype=np.float32)
            cnt = len(rel)
        else:
            acc = norm[m, :].copy()
            cnt = 1 + len(rel)
        for a in rel:
            acc = (acc + norm[a, :]).astype(np.float32)
        new_imp = (acc / np.float32(cnt)).astype(np.float32) if cnt > 0 else acc
        new_rel = _take(new_imp, mode, k, tok, cand_len)
        runs += 1
        if new_rel == rel:
            break
        rel = new_rel
    return [groups[b] for b in rel], runs


# ----------------------------------------------------------------------------
# whole selective prefill
# ----------------------------------------------------------------------------
def keep_prefill(sh: Shape, layers, embed: np.ndarray, token_ids: np.ndarray, group_len: Sequence[int],
                 instr_len: int, k_blocks, v_blocks, ratios: Sequence[float], hops: int,
                 mode: int = BUDGET_GROUP_COUNT, forced_sets: Optional[Sequence[Sequence[int]]] = None,
                 dtype=np.float64):
    """Selective-recompute prefill of the joined prompt.

    k_blocks[l][g], v_blocks[l][g]: group caches at local positions.
    ratios[l]: share of memories recomputed at layer l; ratios[0] is 1 (all) or 0 (none).
    forced_sets: if given, forced_sets[l] replaces the selected set of layer l
    (teacher forcing for parity tests); scores are still computed.

    Returns dict with k_hat[l], v_hat[l] ([N, n_kv_heads, head_dim]), x_final
    [instr_len, hidden], sets[l] (sorted groups recomputed at l), scores[l], hops_run[l].
    """
    n_groups = len(group_len)
    assert ratios[0] in (0.0, 1.0)
    k_hat, v_hat = [], []
    for l in range(sh.n_layers):
        kh, vh = realign_concat(sh, k_blocks[l], v_blocks[l], group_len, instr_len, dtype)
        k_hat.append(kh)
        v_hat.append(vh)
    cur = list(range(n_groups)) if ratios[0] == 1.0 else []
    if forced_sets is not None:
        cur = sorted(forced_sets[0])
    pos = rows_of(cur, group_len, instr_len)
    x = embed[np.asarray(token_ids)[pos]].astype(dtype)
    sets, scores, hops_run = [], [], []
    for l in range(sh.n_layers):
        sets.append(list(cur))
        x, _, s = selective_layer(sh, layers[l], x, cur, group_len, instr_len, k_hat[l], v_hat[l])
        scores.append(s)
        if l + 1 == sh.n_layers:
            hops_run.append(0)
            break
        nxt, runs = select_multihop(s, cur, group_len, ratios[l + 1], hops, mode)
        hops_run.append(runs)
        if forced_sets is not None:
            nxt = sorted(forced_sets[l + 1])
            assert set(nxt) <= set(cur), "relevant sets must be nested"
        # hidden rows of memories that leave the set are discarded
        pos_next = rows_of(nxt, group_len, instr_len)
        keep = np.searchsorted(pos, pos_next)
        x = x[keep]
        cur, pos = nxt, pos_next
    return {"k_hat": k_hat, "v_hat": v_hat, "x_final": x[len(x) - instr_len:], "sets": sets,
            "scores": scores, "hops_run": hops_run}


# ----------------------------------------------------------------------------
# token-granularity recomputation (the comparison scheme of Section 3 and of
# Section 4.2, "System advantage"): tokens, not memories, are the units.  The
# tokens to recompute are chosen by how far their recomputed K/V state lies from
# the cached one, every cached block is loaded in full, and the recomputed
# tokens' K/V are written over the loaded rows in place.
# ----------------------------------------------------------------------------
def token_budget_count(ratio: float, mem_tokens: int, n_candidates: int) -> int:
    """Number of memory tokens to keep: ratio of the prompt's memory tokens, rounded up."""
    k = int(np.ceil(float(np.float32(ratio)) * mem_tokens - BUDGET_EPS))
    return max(0, min(n_candidates, k))


def token_deviation(k_new: np.ndarray, v_new: np.ndarray, k_old: np.ndarray, v_old: np.ndarray) -> np.ndarray:
    """Per token, the squared distance between its recomputed K/V state and its cached
    one (both as they sit in the cache format, keys at the same global position):
    sum over KV heads and head dimensions of (k_new - k_old)^2 + (v_new - v_old)^2.
    Reading: Section 3 speaks of the discrepancy between the full-attention KV state
    and the cached KV state without fixing a norm; the squared Euclidean one is taken.
    Inputs [n, n_kv_heads, head_dim]; returns [n]."""
    dk = (k_new - k_old).reshape(k_new.shape[0], -1)
    dv = (v_new - v_old).reshape(v_new.shape[0], -1)
    return (dk * dk).sum(axis=1) + (dv * dv).sum(axis=1)


def select_tokens(deviation: np.ndarray, k: int) -> List[int]:
    """Indices of the k candidates with the largest deviation (compared as binary32
    values, because they decide integers), the lower index first among equal values;
    returned ascending."""
    d32 = np.asarray(deviation, dtype=np.float32)
    order = sorted(range(len(d32)), key=lambda i: (-float(d32[i]), i))
    return sorted(order[:max(0, k)])


def recompute_token_rows(sh: Shape, w: Dict[str, np.ndarray], x: np.ndarray, pos: np.ndarray,
                         k_hat: np.ndarray, v_hat: np.ndarray):
    """One layer for the token rows at global positions `pos` (ascending; x[n, hidden] holds
    their hidden rows): project, measure the deviation from the cache rows they replace,
    overwrite those rows in place, attend over the whole cache causally, output projection
    and FFN.  Returns (x_out [n, hidden], deviation [n])."""
    q, k, v = project_qkv(sh, w, x, pos)
    k = round_to_storage(k, sh.storage)
    v = round_to_storage(v, sh.storage)
    dev = token_deviation(k, v, k_hat[pos], v_hat[pos])
    k_hat[pos] = k
    v_hat[pos] = v
    n_total = k_hat.shape[0]
    rep = sh.n_q_heads // sh.n_kv_heads
    visible = np.arange(n_total)[None, :] <= pos[:, None]
    o = np.empty_like(q)
    for h in range(sh.n_q_heads):
        s = (q[:, h, :] @ k_hat[:, h // rep, :].T) / np.sqrt(float(sh.head_dim))
        s = np.where(visible, s, -np.inf)
        e = np.exp(s - s.max(axis=1, keepdims=True))
        o[:, h, :] = (e / e.sum(axis=1, keepdims=True)) @ v_hat[:, h // rep, :]
    return output_and_ffn(sh, w, x, o), dev


def keep_prefill_tokens(sh: Shape, layers, embed: np.ndarray, token_ids: np.ndarray, group_len: Sequence[int],
                        instr_len: int, k_blocks, v_blocks, ratios: Sequence[float],
                        forced_rows: Optional[Sequence[Sequence[int]]] = None, dtype=np.float64):
    """Token-granularity selective prefill of the joined prompt.

    Layer l recomputes the memory tokens of T_l and every instruction token; T_0 is every
    memory token (ratios[0] = 1) or none (0).  T_{l+1} = the ceil(ratios[l+1] * N_mem)
    tokens of T_l whose K/V at layer l deviate most from the cache (ties: lower position),
    so the sets are nested as in the memory-granularity method.
    Reading: the deviation of layer l decides layer l+1; at layer 0 it is zero up to rounding
    (K/V of the first layer depend on the token alone), so a schedule that means anything
    keeps ratios[1] = 1 and starts selecting from layer 1's deviation.
    forced_rows[l]: positions of the memory tokens recomputed at layer l (teacher forcing).

    Returns dict with k_hat[l], v_hat[l], x_final [instr_len, hidden], rows[l] (sorted memory
    positions recomputed at l), deviation[l] (aligned with rows[l])."""
    n_mem = int(np.sum(group_len))
    assert ratios[0] in (0.0, 1.0)
    k_hat, v_hat = [], []
    for l in range(sh.n_layers):
        kh, vh = realign_concat(sh, k_blocks[l], v_blocks[l], group_len, instr_len, dtype)
        k_hat.append(kh)
        v_hat.append(vh)
    instr_pos = np.arange(n_mem, n_mem + instr_len, dtype=np.int64)
    cur = np.arange(n_mem, dtype=np.int64) if ratios[0] == 1.0 else np.zeros(0, dtype=np.int64)
    if forced_rows is not None:
        cur = np.asarray(sorted(forced_rows[0]), dtype=np.int64)
    pos = np.concatenate([cur, instr_pos])
    x = embed[np.asarray(token_ids)[pos]].astype(dtype)
    rows, deviations = [], []
    for l in range(sh.n_layers):
        rows.append([int(p) for p in cur])
        x, dev = recompute_token_rows(sh, layers[l], x, pos, k_hat[l], v_hat[l])
        deviations.append(dev[:len(cur)])
        if l + 1 == sh.n_layers:
            break
        if forced_rows is not None:
            nxt = np.asarray(sorted(forced_rows[l + 1]), dtype=np.int64)
            assert set(nxt.tolist()) <= set(cur.tolist()), "token sets must be nested"
            keep = np.searchsorted(cur, nxt)
        else:
            keep = np.asarray(select_tokens(dev[:len(cur)], token_budget_count(ratios[l + 1], n_mem, len(cur))),
                              dtype=np.int64)
            nxt = cur[keep]
        # hidden rows of the tokens that leave the set are discarded
        x = np.concatenate([x[keep], x[len(cur):]])
        cur = nxt
        pos = np.concatenate([cur, instr_pos])
    return {"k_hat": k_hat, "v_hat": v_hat, "x_final": x[len(x) - instr_len:], "rows": rows,
            "deviation": deviations}


# ----------------------------------------------------------------------------
# first token and short greedy decoding over the joined cache
# (Section 1: the planner emits a short action after the long prompt;
#  Section 5: the decoder continues on the cache that `prefill_layer` updated)
# ----------------------------------------------------------------------------
def lm_logits(sh: Shape, final_norm: np.ndarray, lm_head: np.ndarray, x: np.ndarray) -> np.ndarray:
    """Final RMSNorm and vocabulary projection of hidden rows x [n, hidden] -> [n, vocab]."""
    return rmsnorm(x, final_norm, sh.rms_eps) @ lm_head.T


def greedy_token(logits_row: np.ndarray) -> int:
    """reading: greedy decoding, the lowest token id among equal maxima."""
    return int(np.argmax(logits_row))


def decode_layer(sh: Shape, w: Dict[str, np.ndarray], x_row: np.ndarray, position: int,
                 k_cache_l: np.ndarray, v_cache_l: np.ndarray):
    """One new token at `position` through one layer: its K/V go to cache row `position` (rounded to the
    cache format), it attends to rows 0..position, then output projection and FFN.
    k_cache_l, v_cache_l: [rows >= position + 1, n_kv_heads, head_dim], updated in place."""
    x = x_row.reshape(1, -1)
    q, k, v = project_qkv(sh, w, x, np.array([position]))
    k_cache_l[position] = round_to_storage(k, sh.storage)[0]
    v_cache_l[position] = round_to_storage(v, sh.storage)[0]
    rep = sh.n_q_heads // sh.n_kv_heads
    o = np.empty_like(q)
    for h in range(sh.n_q_heads):
        kk = k_cache_l[:position + 1, h // rep, :]
        s = (kk @ q[0, h, :]) / np.sqrt(float(sh.head_dim))
        p = np.exp(s - s.max())
        p = p / p.sum()
        o[0, h, :] = p @ v_cache_l[:position + 1, h // rep, :]
    return output_and_ffn(sh, w, x, o)[0]


def greedy_decode(sh: Shape, layers, embed: np.ndarray, final_norm: np.ndarray, lm_head: np.ndarray,
                  x_last: np.ndarray, k_cache: Sequence[np.ndarray], v_cache: Sequence[np.ndarray], n_ctx: int,
                  n_new: int, forced_tokens: Optional[Sequence[int]] = None, dtype=np.float64):
    """n_new greedy tokens after a prompt of n_ctx tokens whose last hidden row is x_last.

    Token 0 comes from x_last; token t > 0 from running token t-1 at position n_ctx + t - 1 through every
    layer over the cache (which gains that token's K/V).  forced_tokens[t], if given, replaces the choice
    fed forward (teacher forcing for parity tests); the logits are those of the free choice either way.
    k_cache[l], v_cache[l]: [rows >= n_ctx + n_new - 1, n_kv_heads, head_dim], updated in place.
    Returns (tokens [n_new], logits [n_new, vocab])."""
    tokens, logits = [], []
    x = np.asarray(x_last, dtype=dtype)
    for t in range(n_new):
        lg = lm_logits(sh, final_norm, lm_head, x.reshape(1, -1))[0]
        logits.append(lg)
        tok = greedy_token(lg)
        tokens.append(tok)
        if t + 1 == n_new:
            break
        fed = tok if forced_tokens is None else int(forced_tokens[t])
        x = embed[fed].astype(dtype)
        for l in range(sh.n_layers):
            x = decode_layer(sh, layers[l], x, n_ctx + t, k_cache[l], v_cache[l])
    return tokens, np.stack(logits)
