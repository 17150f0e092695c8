"""Pins of the static-dynamic memory oracle (Section 4.1): none of them re-types its rule."""
import json
import os

import numpy as np
import pytest

from oracle.memory_oracle import DYNAMIC, STATIC, MemoryOracle

HERE = os.path.dirname(__file__)


def run_trace(make, trace):
    """Drive a store through a trace of steps; yields (expected, report, units) per step."""
    m = make(trace["window_t"])
    for st in trace["steps"]:
        for op in st["ops"]:
            if op[0] == "put":
                m.put(op[1], op[2], op[3])
            else:
                m.remove(op[1])
        rep = m.end_step()
        units = m.units()
        yield st["expect"], rep, units
        for u in units:
            if u.dirty:
                m.mark_computed(u)


def test_hand_worked_trace():
    trace = json.load(open(os.path.join(HERE, "golden", "memory_trace_t3.json")))
    for i, (exp, rep, units) in enumerate(run_trace(MemoryOracle, trace)):
        assert rep.step == i
        got = dict(n_static=rep.n_static, n_dynamic=rep.n_dynamic, to_dynamic=rep.to_dynamic, to_static=rep.to_static,
                   dirty_units=rep.dirty_units, dirty_tokens=rep.dirty_tokens,
                   units=[[u.kind, u.ident, u.n_tokens] for u in units])
        assert got == exp, "step %d" % i


def random_ops(rng, live, n_groups, max_seg):
    """A few random changes for one step; `live` maps segment -> group."""
    ops = []
    for _ in range(rng.integers(0, 3)):
        r = rng.random()
        if r < 0.55 or not live:
            g = int(rng.integers(0, n_groups))
            cand = [s for s, gg in live.items() if gg == g]
            if cand and rng.random() < 0.6:
                s = int(rng.choice(cand))
            else:
                s = int(rng.integers(0, max_seg)) * n_groups + g     # ids of different groups never collide
            toks = [int(x) for x in rng.integers(0, 50, size=rng.integers(1, 6))]
            ops.append(("put", g, s, toks))
            live[s] = g
        elif r < 0.7:
            s = int(rng.choice(list(live)))
            ops.append(("remove", s))
            del live[s]
    return ops


@pytest.mark.parametrize("t", [0, 1, 2, 4, 10])
def test_classification_matches_the_sentence_on_a_change_log(t):
    """Static <=> nothing about the group changed during the recent t steps, read off a full
    log of change events (set scan), not off the store's own bookkeeping."""
    rng = np.random.default_rng(100 + t)
    m = MemoryOracle(t)
    live, content, log = {}, {}, []           # log: (step, group)
    for step in range(60):
        for op in random_ops(rng, live, 4, 5):
            if op[0] == "put":
                _, g, s, toks = op
                if content.get(s) != tuple(toks):
                    log.append((step, g))
                content[s] = tuple(toks)
                m.put(g, s, toks)
            else:
                s = op[1]
                g = m.seg[s].group
                log.append((step, g))
                del content[s]
                m.remove(s)
        m.end_step()
        recent = set(range(step - t + 1, step + 1))
        for gid, grp in m.grp.items():
            changed = any(st in recent for st, g in log if g == gid)
            assert grp.kind == (DYNAMIC if changed else STATIC), (step, gid)


def test_update_of_a_dynamic_segment_invalidates_that_segment_only():
    m = MemoryOracle(10)
    for s in range(5):
        m.put(0, s, [s] * (s + 2))
    m.end_step()
    for u in m.units():
        m.mark_computed(u)
    m.put(0, 3, [9, 9, 9])
    rep = m.end_step()
    assert rep.dirty_units == 1 and rep.dirty_tokens == 3
    assert [u.ident for u in m.units() if u.dirty] == [3]


def test_update_inside_a_static_group_recomputes_every_segment_on_its_own():
    m = MemoryOracle(2)
    lens = [3, 4, 5]
    for s, n in enumerate(lens):
        m.put(7, s, list(range(n)))
    reps = [m.end_step() for _ in range(3)]           # ages 0, 1, 2 -> static at the third close
    assert [r.to_static for r in reps] == [[], [], [7]]
    (u,) = m.units()
    assert (u.kind, u.ident, u.n_tokens, u.dirty) == (STATIC, 7, sum(lens), True)
    assert m.unit_tokens(u) == [0, 1, 2, 0, 1, 2, 3, 0, 1, 2, 3, 4]   # segments in id order, jointly cached
    m.mark_computed(u)
    assert m.end_step().dirty_tokens == 0
    m.put(7, 1, [8])
    rep = m.end_step()
    assert rep.to_dynamic == [7]
    units = m.units()
    assert [(x.kind, x.ident, x.n_tokens, x.dirty) for x in units] == [(DYNAMIC, 0, 3, True), (DYNAMIC, 1, 1, True),
                                                                       (DYNAMIC, 2, 5, True)]
    assert rep.dirty_tokens == 9


def test_identical_content_is_no_change_and_window_zero_is_all_static():
    m = MemoryOracle(0)
    assert m.put(1, 1, [1, 2]) is True
    assert m.put(1, 1, [1, 2]) is False
    rep = m.end_step()
    assert rep.n_static == 1 and rep.to_static == [1]
    m2 = MemoryOracle(1)
    m2.put(0, 0, [5])
    m2.end_step()
    assert m2.put(0, 0, [5]) is False
    rep = m2.end_step()
    assert rep.to_static == [0]                       # the rewrite did not restart the window


def test_stable_groups_change_category_once_per_window():
    """Section 4.1: a category change 'happens at a low frequency'.  With one update every p > t
    steps a group flips to static and back once per update, never more."""
    t, p = 3, 8
    m = MemoryOracle(t)
    m.put(0, 0, [1])
    flips = 0
    for step in range(64):
        if step % p == 0:
            m.put(0, 0, [step + 2])
        rep = m.end_step()
        flips += len(rep.to_static) + len(rep.to_dynamic)
        for u in m.units():
            m.mark_computed(u)
    assert flips == 2 * (64 // p) - 1          # the very first step starts dynamic: no flip into it
