"""Pins of the oracle's integer logic: units, groups, visiting order, parameter counts."""
import json
import os

import numpy as np
import pytest

from hift_inputs import WORKLOADS, model_config
from oracle import hift_oracle as O

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))


def test_units_and_groups_printed_in_paper():
    cfg = model_config(WORKLOADS["C4"])
    assert O.n_units(cfg) == GOLD["llama7b_units"]["value"]
    assert O.n_groups(O.n_units(cfg), 1) == GOLD["llama7b_groups_m1"]["value"]


@pytest.mark.parametrize("n,m,k", [(4, 1, 4), (14, 1, 14), (26, 2, 13), (34, 1, 34), (42, 4, 11),
                                   (42, 1, 42), (5, 5, 1), (5, 7, 1), (7, 2, 4)])
def test_group_count_rule(n, m, k):
    # k = n/m if m | n else floor(n/m)+1, written out independently here
    assert O.n_groups(n, m) == k
    units = [u for j in range(k) for u in O.group_units(n, m, j)]
    assert units == list(range(n))                      # consecutive, disjoint, complete
    assert all(len(O.group_units(n, m, j)) == m for j in range(k - 1))
    assert 1 <= len(O.group_units(n, m, k - 1)) <= m    # the short group is the top one


def test_13b_group_layout_m4():
    assert O.group_units(42, 4, 10) == [40, 41]


def test_orders():
    for k in (1, 2, 11, 34):
        b = O.group_order(k, "bottom2up")
        t = O.group_order(k, "top2down")
        r = O.group_order(k, "random", 12345)
        assert b == list(range(k)) and t == b[::-1]
        assert sorted(r) == b                            # each group once per cycle
        assert r == O.group_order(k, "random", 12345)    # drawn once, reproducible
    assert O.group_order(34, "random", 1) != O.group_order(34, "random", 2)


def test_splitmix64_published_vectors():
    # first outputs for seed 1234567 from the reference implementation's published test vector
    s = 1234567
    outs = []
    for _ in range(5):
        v, s = O.splitmix64(s)
        outs.append(v)
    assert outs == [6457827717110365317, 3203168211198807973, 9817491932198370423,
                    4593380528125082431, 16408922859458223821]


def test_schedule_is_periodic_and_cycles():
    cfg = model_config(WORKLOADS["C1"])
    o = O.HiftOracle(cfg, WORKLOADS["C1"]["opt"], np.zeros(O.n_params(cfg)))
    k = o.set_group_schedule("random", 1, 7)
    seq = [o.schedule_group_at(t) for t in range(1, 3 * k + 1)]
    assert seq[:k] == seq[k:2 * k] == seq[2 * k:]
    assert sorted(seq[:k]) == list(range(k))


@pytest.mark.parametrize("name,layer,emb,head,total", [
    ("C1", 49984, 18432, 16512, 18432 + 2 * 49984 + 16512),
    ("C2", 7087872, 38999808, 1538, 38999808 + 12 * 7087872 + 1538),
    ("C4", 202383360, 131072000, 131076096, 6738415616),
    ("C5", 317204480, 163840000, 163845120, 163840000 + 40 * 317204480 + 163845120),
])
def test_param_counts(name, layer, emb, head, total):
    cfg = model_config(WORKLOADS[name])
    ur = O.unit_ranges(cfg)
    assert ur[0][1] == emb and ur[1][1] == layer and ur[-1][1] == head
    assert O.n_params(cfg) == total
    assert all(ur[i][0] + ur[i][1] == ur[i + 1][0] for i in range(len(ur) - 1))


def test_peak_trainable_share_13b():
    cfg = model_config(WORKLOADS["C5"])
    ur = O.unit_ranges(cfg)
    share = 100.0 * max(c for _o, c in ur) / O.n_params(cfg)
    g = GOLD["peak_trainable_share_13b_percent"]
    assert abs(share - g["value"]) <= g["tol"]


def test_memory_closed_forms_equal_groups():
    # fp32 AdamW, equal-size groups: resident P + G + S = (k+3)/k * P  (hift), 4 P (fpft)
    P, k = 1200, 12
    grp = P // k
    assert P + 2 * P + P == GOLD["memory_fpft_over_zeta1"]["value"] * P
    assert P + 2 * grp + grp == (k + 3) * P // k


def test_memory_model_against_the_printed_forms():
    """The oracle's accounting reduces to the appendix's three equations for fp32 AdamW and to the
    worked FPFT figure; for other optimizers only the state multiplicity changes."""
    from fractions import Fraction
    cfg = model_config(WORKLOADS["C4"])
    mm = O.memory_model(cfg, 1)
    k = GOLD["llama7b_groups_m1"]["value"]
    assert mm["k"] == k
    assert mm["zeta_fpft"] == GOLD["memory_fpft_over_zeta1"]["value"] * mm["zeta1"]
    assert abs(mm["zeta_hift"] - float(Fraction(k + 3, k)) * mm["zeta1"]) <= 1e-6 * mm["zeta1"]
    assert abs(mm["delta"] - float(Fraction(3 * k - 3, k)) * mm["zeta1"]) <= 1e-6 * mm["zeta1"]
    w = GOLD["memory_fpft_7b_worked"]
    assert abs(w["fpft_G"] - 4 * w["zeta1_G"]) < 1e-9          # the printed pair obeys the first equation
    # the peak uses the largest group (a hidden layer at 7B), the average an equal share
    layer = max(c for _o, c in O.unit_ranges(cfg))
    assert mm["peak_trainable"] == layer and mm["zeta_hift_peak"] == mm["zeta1"] + 12 * layer
    assert mm["zeta_hift_peak"] >= mm["zeta_hift"]
    # plain SGD keeps no state: gradients are the only extra term
    sgd = O.memory_model(cfg, 1, state_arrays=0)
    assert sgd["zeta_fpft"] == 2 * sgd["zeta1"] and sgd["zeta_hift_peak"] == sgd["zeta1"] + 4 * layer
    # grouping m units: k shrinks, the peak group grows
    m4 = O.memory_model(cfg, 4)
    assert m4["k"] == 9 and m4["peak_trainable"] == 4 * layer
