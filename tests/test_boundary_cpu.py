"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad descriptions before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2602_23592_amd import binding as kb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    names = set()
    inc = os.path.join(ROOT, "include")
    for h in sorted(os.listdir(inc)):
        if not h.endswith(".h"):
            continue
        text = open(os.path.join(inc, h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(keep_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = kb.load_library()
    names = _declared_functions()
    assert {"keep_init", "keep_score_groups", "keep_recompute_layer", "keep_prefill"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(kb.EXPORTED) == names


def _desc(**kw):
    base = dict(n_layers=2, hidden=64, n_q_heads=4, n_kv_heads=2, head_dim=16, ffn_dim=96, vocab=97,
                rope_theta=1e4, rms_eps=1e-6, dtype=kb.KEEP_F32, max_tokens=128, max_groups=8, kernel_path=0)
    base.update(kw)
    return kb.ModelDesc(*[base[f[0]] for f in kb.ModelDesc._fields_])


def _init(desc, layers_ok=True):
    lib = kb.load_library()
    arr = (kb.LayerWeights * 2)()
    if layers_ok:
        for l in range(2):
            for n in ("ln1", "wq", "wk", "wv", "wo", "ln2", "wgate", "wup", "wdown"):
                setattr(arr[l], n, 0x1000)          # never dereferenced: validation comes first
    h = C.c_void_p()
    st = lib.keep_init(C.byref(desc) if desc is not None else None, arr, 0x1000, None, None, None, C.byref(h))
    return st, lib.keep_last_error(None).decode(), h


@pytest.mark.parametrize("kw,status", [
    (dict(n_layers=0), kb.KEEP_ERR_INVALID_ARG),
    (dict(n_q_heads=5), kb.KEEP_ERR_INVALID_ARG),            # not a multiple of n_kv_heads
    (dict(dtype=7), kb.KEEP_ERR_INVALID_ARG),
    (dict(kernel_path=3), kb.KEEP_ERR_INVALID_ARG),
    (dict(rope_theta=0.0), kb.KEEP_ERR_INVALID_ARG),
    (dict(max_tokens=0), kb.KEEP_ERR_INVALID_ARG),
    (dict(head_dim=24), kb.KEEP_ERR_SHAPE),                  # not a multiple of 16
    (dict(head_dim=512), kb.KEEP_ERR_SHAPE),
    (dict(hidden=60), kb.KEEP_ERR_SHAPE),
    (dict(n_layers=129), kb.KEEP_ERR_SHAPE),
])
def test_keep_init_rejects_bad_descriptions(kw, status):
    st, text, h = _init(_desc(**kw))
    assert st == status and text and not h.value


def test_keep_init_null_arguments():
    lib = kb.load_library()
    st, text, h = _init(None)
    assert st == kb.KEEP_ERR_INVALID_ARG and "NULL" in text
    st, text, h = _init(_desc(), layers_ok=False)
    assert st == kb.KEEP_ERR_INVALID_ARG and "weight pointer" in text
    assert lib.keep_init(C.byref(_desc()), None, None, None, None, None, None) == kb.KEEP_ERR_INVALID_ARG
    assert lib.keep_destroy(None) == kb.KEEP_OK
    assert lib.keep_uses_mfma(None) == -1


def test_workspace_bytes_scale_with_the_description():
    lib = kb.load_library()
    small = lib.keep_workspace_bytes(C.byref(_desc()))
    big = lib.keep_workspace_bytes(C.byref(_desc(max_tokens=4096)))
    assert 0 < small < big
    assert lib.keep_workspace_bytes(C.byref(_desc(head_dim=24))) == 0
    assert lib.keep_workspace_bytes(None) == 0


def test_calls_on_a_null_context_fail_cleanly():
    lib = kb.load_library()
    assert lib.keep_recompute_layer(None, None, 0, None, 0, None, None, None, None) == kb.KEEP_ERR_INVALID_ARG
    assert lib.keep_score_groups(None, None, 0, None, 0, 0.5, 1, 0, None, None, None, None) == kb.KEEP_ERR_INVALID_ARG
    assert lib.keep_select_groups(None, None, None, 0, None, 0, 0.5, 1, 0, None, None, None) == kb.KEEP_ERR_INVALID_ARG
    assert lib.keep_prefill(None, None, None, 1, 0, 0, None, None, None, None, None, None) == kb.KEEP_ERR_INVALID_ARG


def test_workload_recipes_are_exact_and_seeded():
    import numpy as np
    import keep_synth as ks
    for name, w in ks.WORKLOADS.items():
        a, ka = ks.group_lengths(w)
        b, _ = ks.group_lengths(w)
        assert np.array_equal(a, b) and int(a.sum()) == w.mem_tokens and len(ka) == len(a)
        lo = min(r[1] for r in w.group_recipe)
        hi = max(r[2] for r in w.group_recipe)
        assert a.min() >= lo and a.max() <= hi
    r = ks.ratio_schedule(0.1, 48)
    assert r[0] == 1.0 and abs(float(np.mean(r[1:])) - 0.1) < 1e-6 and all(r[i] >= r[i + 1] for i in range(1, 47))
    assert np.allclose(ks.ratio_schedule(0.15, 2), [1.0, 0.15])
