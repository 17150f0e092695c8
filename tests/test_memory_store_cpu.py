"""The library's static-dynamic memory store (host code behind the C ABI) against the oracle of
Section 4.1: same traces, every report field, unit list and unit content equal at every step."""
import json
import os

import numpy as np
import pytest

from oracle.memory_oracle import MemoryOracle
from paper_2602_23592_amd import KeepError, KeepMemory
from test_memory_oracle import random_ops

HERE = os.path.dirname(__file__)


def compare_step(lib_mem, ora, step):
    rep, to_dyn, to_sta = lib_mem.end_step()
    orep = ora.end_step()
    assert (rep.step, rep.n_static, rep.n_dynamic, rep.dirty_units, rep.dirty_tokens) == \
           (orep.step, orep.n_static, orep.n_dynamic, orep.dirty_units, orep.dirty_tokens), step
    assert to_dyn == orep.to_dynamic and to_sta == orep.to_static, step
    units, ounits = lib_mem.units(), ora.units()
    assert [(u.kind, u.id, u.n_segments, u.n_tokens, u.dirty) for u in units] == \
           [(u.kind, u.ident, len(u.segments), u.n_tokens, int(u.dirty)) for u in ounits], step
    for i, (u, ou) in enumerate(zip(units, ounits)):
        assert lib_mem.unit_tokens(i, u.n_tokens) == ora.unit_tokens(ou), (step, i)
    return units, ounits


@pytest.mark.parametrize("t,seed,mark", [(0, 1, 1.0), (1, 2, 1.0), (3, 3, 0.5), (10, 4, 1.0), (10, 5, 0.0), (4, 6, 0.7)])
def test_random_traces_match_the_oracle(t, seed, mark):
    rng = np.random.default_rng(seed)
    lib_mem, ora = KeepMemory(t), MemoryOracle(t)
    live = {}
    for step in range(80):
        for op in random_ops(rng, live, 5, 6):
            if op[0] == "put":
                assert lib_mem.put(op[1], op[2], op[3]) == ora.put(op[1], op[2], op[3])
            else:
                lib_mem.remove(op[1])
                ora.remove(op[1])
        units, ounits = compare_step(lib_mem, ora, step)
        for i, (u, ou) in enumerate(zip(units, ounits)):      # the caller computes some or all stale units
            if u.dirty and rng.random() < mark:
                lib_mem.mark_computed(i)
                ora.mark_computed(ou)
    lib_mem.close()


def test_hand_worked_trace_through_the_library():
    trace = json.load(open(os.path.join(HERE, "golden", "memory_trace_t3.json")))
    m = KeepMemory(trace["window_t"])
    for i, st in enumerate(trace["steps"]):
        for op in st["ops"]:
            if op[0] == "put":
                m.put(op[1], op[2], op[3])
            else:
                m.remove(op[1])
        rep, to_dyn, to_sta = m.end_step()
        units = m.units()
        got = dict(n_static=rep.n_static, n_dynamic=rep.n_dynamic, to_dynamic=to_dyn, to_static=to_sta,
                   dirty_units=rep.dirty_units, dirty_tokens=rep.dirty_tokens,
                   units=[[u.kind, u.id, u.n_tokens] for u in units])
        assert got == st["expect"], "step %d" % i
        for j, u in enumerate(units):
            if u.dirty:
                m.mark_computed(j)


def test_error_paths():
    m = KeepMemory(2)
    m.put(0, 0, [1, 2, 3])
    with pytest.raises(KeepError):
        m.put(1, 0, [4])                 # the segment belongs to group 0
    with pytest.raises(KeepError):
        m.put(0, 1, [])                  # empty segment
    with pytest.raises(KeepError):
        m.remove(99)
    with pytest.raises(KeepError):
        m.unit_tokens(0, 2)              # capacity too small
    with pytest.raises(KeepError):
        m.mark_computed(5)
    with pytest.raises(KeepError):
        KeepMemory(-1)
