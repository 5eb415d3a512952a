"""CPU-only checks of the C-ABI library: it loads, exports every function include/hift.h declares,
and its host-side integer logic (layout, groups, orders, arena sizes, argument errors) agrees with
the oracle.  No kernel is launched here."""
import os
import re

import numpy as np
import pytest

from hift_inputs import WORKLOADS, model_config
from oracle import hift_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def H():
    import paper_2401_15207_amd as H
    return H


def declared_functions():
    text = open(os.path.join(ROOT, "include", "hift.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hift_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(H):
    names = declared_functions()
    assert len(names) >= 25 and "hift_step" in names and "hift_model_create" in names
    missing = [n for n in names if not hasattr(H.lib, n)]
    assert not missing, missing


def test_layout_matches_oracle_for_all_workloads(H):
    cfgs = [model_config(WORKLOADS[name]) for name in ("C1", "C2", "C3", "C4", "C5", "C4_L2", "C5_L2")]
    cfgs += [model_config(WORKLOADS[name], tie_embeddings=1) for name in ("C1", "C4")]     # no whead tensor
    assert O.n_params(cfgs[-1]) == O.n_params(cfgs[3]) - 32000 * 4096
    with pytest.raises(H.HiftError):
        H.tensor_list(model_config(WORKLOADS["C2"], tie_embeddings=1))                        # the encoder has no output matrix to tie
    for cfg in cfgs:
        tl, n = H.tensor_list(cfg)
        ref = O.param_tensors(cfg)
        assert n == O.n_params(cfg) and len(tl) == len(ref)
        off = 0
        for (gn, gs, gk, gu, go), (rn, rs, rk, ru) in zip(tl, ref):
            assert (gn, tuple(gs), gk, gu, go) == (rn, tuple(rs), rk, ru, off)
            off += int(np.prod(rs))


def test_groups_and_orders_match_oracle(H):
    for n in (4, 14, 26, 34, 42):
        for m in (1, 2, 3, 4, 5, n, n + 3):
            k = H.group_count(n, m)
            assert k == O.n_groups(n, m)
            for s in ("bottom2up", "top2down", "random"):
                for seed in (0, 1, 2 ** 63 + 5):
                    assert H.group_order(k, s, seed) == O.group_order(k, s, seed)


def test_arena_sizes(H):
    wl = WORKLOADS["C4"]
    cfg = model_config(wl)
    n = O.n_params(cfg)
    big = max(c for _o, c in O.unit_ranges(cfg))
    d_host, p_host = H.query_bytes(dict(cfg, state_on_host=1), wl["opt"], 1, 4, 512)
    d_res, p_res = H.query_bytes(dict(cfg, state_on_host=0), wl["opt"], 1, 4, 512)
    assert p_res == 0 and p_host == 2 * 4 * n                       # AdamW: m and v of every parameter
    assert d_res - d_host >= 2 * 4 * (n - 3 * big) - 4096            # three slots (in use, arriving, draining) instead of all state
    sgd = dict(kind="sgd", lr=0.1, momentum=0.0, weight_decay=0.0)
    _d, p = H.query_bytes(dict(cfg, state_on_host=1), sgd, 1, 4, 512)
    assert p == 0                                                    # plain SGD keeps no state
    # fp32 AdamW, equal groups: parameters + gradient + state slots per group = (k+3)/k of the parameters
    # (appendix "Memory Analysis"); here the largest group of the 7B shape is one layer
    assert 4 * big + 2 * 4 * big == 3 * 4 * big


def test_memory_report(H):
    wl = WORKLOADS["C4"]
    cfg = model_config(wl)
    ref = O.memory_model(cfg, 1)
    base = H.memory_report(dict(cfg, state_on_host=1), wl["opt"], 1, 4, 512)
    d, p = H.query_bytes(dict(cfg, state_on_host=1), wl["opt"], 1, 4, 512)
    assert base["device_total"] == d and base["pinned_total"] == p
    parts = ["device_master", "device_forward", "device_packed", "device_grad", "device_state", "device_activations",
             "device_workspace"]
    assert sum(base[q] for q in parts) == base["device_total"] == base["total"]
    assert base["pgs"] == base["para"] + base["gra"] + base["sta"] and base["total"] == base["pgs"] + base["residual"]
    # closed forms (appendix "Memory Analysis") against the oracle's
    for key in ("k", "n_params", "peak_trainable"):
        assert base[key] == ref[key]
    for key in ("zeta1", "zeta_fpft", "zeta_hift", "zeta_hift_peak"):
        assert abs(base[key] - ref[key]) <= 1e-9 * ref[key]
    # what the arena holds: fp32 master and bf16 copy of every parameter, one gradient buffer and three
    # state slots for the largest group (rounded up to 64 parameters, 256-byte pieces)
    n, big = ref["n_params"], ref["peak_trainable"]
    assert 4 * n <= base["device_master"] < 4 * n + 4096
    # the bf16 copy: every tensor but the matrices that live in their two fragment-order copies (here: all but the
    # token table and the 65 gain vectors)
    plain = 32000 * 4096 + 65 * 4096
    assert 2 * plain <= base["device_forward"] < 2 * plain + 4096
    assert 4 * big <= base["device_grad"] < 4 * big + 4096
    assert 3 * 8 * big <= base["device_state"] < 3 * 8 * big + 4096
    assert base["device_packed"] >= 2 * 2 * (n - 2 * 32000 * 4096 - 300000)   # two copies of every layer matrix and the head
    # the small-memory mode: master of inactive groups on the host, no fragment-order copies
    lean = H.memory_report(dict(cfg, state_on_host=1, master_on_host=1, no_packed_copies=1), wl["opt"], 1, 4, 512)
    assert lean["device_packed"] == 0 and 3 * 4 * big <= lean["device_master"] < 3 * 4 * big + 4096
    assert 2 * n <= lean["device_forward"] < 2 * n + 4096      # without fragment-order copies the bf16 model is whole
    assert lean["pinned_total"] == 12 * n                       # master, m and v of every parameter
    assert lean["device_activations"] == base["device_activations"]
    one = H.memory_report(dict(cfg, state_on_host=1, master_on_host=1, no_packed_copies=1), wl["opt"], 1, 1, 512)
    assert one["device_total"] < 24 * 2 ** 30                   # a 7B model in a 24 GiB budget at batch 1 (appendix "Mixing Precision")
    # all state resident: the state term is the whole of zeta2
    res = H.memory_report(dict(cfg, state_on_host=0), wl["opt"], 1, 4, 512)
    assert 8 * n <= res["device_state"] < 8 * n + 4096 and res["pinned_total"] == 0
    with pytest.raises(H.HiftError):
        H.memory_report(dict(cfg, state_on_host=0, master_on_host=1), wl["opt"], 1, 4, 512)
    with pytest.raises(H.HiftError):
        H.memory_report(dict(cfg, dtype=0, state_on_host=1, master_on_host=1), wl["opt"], 1, 4, 512)


def test_adafactor_keeps_a_few_numbers_per_row_and_column(H):
    wl = WORKLOADS["C4"]
    cfg = model_config(wl)
    af = dict(kind="adafactor", lr=1e-3, weight_decay=0.0)
    r = H.memory_report(dict(cfg, state_on_host=1), af, 1, 4, 512)
    want = sum((s[0] + s[1]) if len(s) >= 2 else s[0] for _n, s, _k, _u in O.param_tensors(cfg))
    assert 4 * want <= r["sta"] < 4 * want + 4096 and r["pinned_total"] == 0
    assert r["sta"] < 1e-3 * r["device_master"]          # against 2 x the weights for AdamW


def test_argument_errors_without_a_gpu(H):
    import ctypes as C
    from paper_2401_15207_amd import binding as B
    k = C.c_int32()
    assert H.lib.hift_group_count(0, 1, C.byref(k)) == -1
    assert H.lib.hift_group_count(4, 0, C.byref(k)) == -1
    assert b"must be" in H.lib.hift_last_error()
    bad = B.make_config(dict(model_config(WORKLOADS["C1"]), n_heads=5))
    n, t = C.c_int32(), C.c_int64()
    assert H.lib.hift_tensor_count(C.byref(bad), C.byref(n), C.byref(t)) == -1
    bad = B.make_config(dict(model_config(WORKLOADS["C1"]), arch=7))
    assert H.lib.hift_tensor_count(C.byref(bad), C.byref(n), C.byref(t)) == -1
    with pytest.raises(H.HiftError):
        H.query_bytes(model_config(WORKLOADS["C1"]), WORKLOADS["C1"]["opt"], 1, 2, 64)   # seq above the position table
    assert H.lib.hift_step(None, None, 0, None) == -1
    assert H.lib.hift_read_params(None, 0, 1, 0, None, 0) == -1
    H.lib.hift_model_destroy(None)
