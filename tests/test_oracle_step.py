"""Pins of the oracle's step logic: masked update (Eq. 2-3), single group == full step
(Eq. 1), hand-computed optimizer updates, delayed learning-rate bookkeeping."""
import numpy as np
import pytest

from hift_inputs import WORKLOADS, init_params, make_batch, model_config
from oracle import hift_oracle as O

WL = WORKLOADS["C1"]
CFG = model_config(WL)
SPEC = [(n, s, k) for n, s, k, _u in O.param_tensors(CFG)]


def _fresh(opt=None, seed=1):
    theta = init_params(seed, SPEC, False, jitter=0.05).astype(np.float64)
    return O.HiftOracle(CFG, opt or WL["opt"], theta), theta


@pytest.mark.parametrize("strategy", ["bottom2up", "top2down", "random"])
def test_frozen_parameters_bit_identical(strategy):
    o, _ = _fresh()
    k = o.set_group_schedule(strategy, 1, 99)
    for t in range(1, 2 * k + 1):
        gid = o.schedule_group_at(t)
        before = o.theta.copy()
        s1, s2 = o.state1.copy(), o.state2.copy()
        tok, lab = make_batch(WL, 1, t)
        o.step(tok, lab, gid)
        lo, hi = o.group_range(gid)
        keep = np.ones(o.theta.size, bool)
        keep[lo:hi] = False
        assert np.array_equal(before[keep], o.theta[keep])
        assert np.array_equal(s1[keep], o.state1[keep]) and np.array_equal(s2[keep], o.state2[keep])
        assert not np.array_equal(before[lo:hi], o.theta[lo:hi])
    assert o.cycles_done == 2


def test_single_group_equals_full_finetuning_step():
    # m = n -> k = 1 -> beta = 1: a plain AdamW step on all parameters, written out here
    o, theta0 = _fresh()
    assert o.set_group_schedule("bottom2up", O.n_units(CFG), 0) == 1
    tok, lab = make_batch(WL, 1, 1)
    o.step(tok, lab, 0)
    _loss, g = O.loss_and_grad(CFG, theta0, tok, lab)
    p = WL["opt"]
    m = (1 - p["beta1"]) * g
    v = (1 - p["beta2"]) * g * g
    th = theta0 * (1 - p["lr"] * p["weight_decay"] * o.decay_mask)
    th = th - p["lr"] * (m / (1 - p["beta1"])) / (np.sqrt(v / (1 - p["beta2"])) + p["eps"])
    assert np.array_equal(th, o.theta)


def test_union_of_group_gradients_is_the_full_gradient():
    # SGD, lr 1, no momentum, no decay: theta0 - theta1 = gradient of the active group
    sgd = dict(kind="sgd", lr=1.0, beta1=0, beta2=0, eps=0, weight_decay=0.0, momentum=0.0)
    tok, lab = make_batch(WL, 1, 1)
    _o, theta0 = _fresh(sgd)
    _loss, g = O.loss_and_grad(CFG, theta0, tok, lab)
    got = np.zeros_like(g)
    for gid in range(4):
        o, _ = _fresh(sgd)
        o.set_group_schedule("bottom2up", 1, 0)
        o.step(tok, lab, gid)
        lo, hi = o.group_range(gid)
        got[lo:hi] = (theta0 - o.theta)[lo:hi]
    assert np.allclose(got, g, rtol=0, atol=1e-15)


def test_adamw_two_steps_by_hand():
    th, m, v = np.array([1.0, -2.0]), np.zeros(2), np.zeros(2)
    dm = np.array([1.0, 0.0])
    g1, g2 = np.array([0.5, -0.25]), np.array([-1.0, 0.125])
    lr, b1, b2, eps, wd = 0.1, 0.9, 0.999, 1e-8, 0.01
    O.adamw_update(th, g1, m, v, 1, lr, b1, b2, eps, wd, dm)
    # step 1 from zero state: theta(1 - lr wd) - lr g/(|g| + eps)
    e1 = np.array([1.0 * (1 - 0.001) - 0.1 * 0.5 / (0.5 + 1e-8), -2.0 + 0.1 * 0.25 / (0.25 + 1e-8)])
    assert np.allclose(th, e1, rtol=1e-14, atol=0)
    O.adamw_update(th, g2, m, v, 2, lr, b1, b2, eps, wd, dm)
    m2 = np.array([0.9 * 0.05 + 0.1 * -1.0, 0.9 * -0.025 + 0.1 * 0.125])
    v2 = np.array([0.999 * 0.00025 + 0.001 * 1.0, 0.999 * 0.0000625 + 0.001 * 0.015625])
    e2 = e1 * np.array([1 - 0.001, 1.0]) - 0.1 * (m2 / (1 - 0.81)) / (np.sqrt(v2 / (1 - 0.998001)) + 1e-8)
    assert np.allclose(m, m2, rtol=1e-14) and np.allclose(v, v2, rtol=1e-14)
    assert np.allclose(th, e2, rtol=1e-13, atol=0)


def test_adagrad_and_sgd_momentum_by_hand():
    th, acc = np.array([1.0]), np.zeros(1)
    O.adagrad_update(th, np.array([0.5]), acc, 0.1, 1e-10, 0.0, np.ones(1))
    assert np.allclose(th, 1.0 - 0.1 * 0.5 / (0.5 + 1e-10), rtol=1e-15) and acc[0] == 0.25
    O.adagrad_update(th, np.array([-1.0]), acc, 0.1, 1e-10, 0.0, np.ones(1))
    assert np.allclose(acc, 1.25) and np.allclose(th, 0.9 + 0.1 / (np.sqrt(1.25) + 1e-10), rtol=1e-9)
    th, buf = np.array([1.0]), np.zeros(1)
    O.sgd_update(th, np.array([0.5]), buf, 1, 0.1, 0.9, 0.0, np.ones(1))
    assert buf[0] == 0.5 and np.allclose(th, 0.95)
    O.sgd_update(th, np.array([0.25]), buf, 2, 0.1, 0.9, 0.0, np.ones(1))
    assert np.allclose(buf, 0.9 * 0.5 + 0.25) and np.allclose(th, 0.95 - 0.07)
    th = np.array([1.0])
    O.sgd_update(th, np.array([0.5]), np.zeros(1), 1, 0.1, 0.0, 0.0, np.ones(1))
    assert np.allclose(th, 0.95)


def test_adagrad_and_sgd_weight_decay_by_hand():
    # L2 decay enters the gradient before anything else: g' = g + wd * theta, on decayed elements only
    th, acc = np.array([2.0, 2.0]), np.zeros(2)
    O.adagrad_update(th, np.array([0.5, 0.5]), acc, 0.1, 1e-10, 0.25, np.array([1.0, 0.0]))
    # element 0: g' = 0.5 + 0.25 * 2 = 1.0, acc = 1.0, step = 0.1 * 1 / (1 + 1e-10); element 1: as without decay
    assert acc[0] == 1.0 and acc[1] == 0.25
    assert np.allclose(th, [2.0 - 0.1 / (1.0 + 1e-10), 2.0 - 0.1 * 0.5 / (0.5 + 1e-10)], rtol=1e-15)
    O.adagrad_update(th, np.array([-1.0, 0.0]), acc, 0.1, 1e-10, 0.25, np.array([1.0, 0.0]))
    g2 = -1.0 + 0.25 * 1.9                       # theta after the first step is 1.9 to 1e-11
    assert np.allclose(acc[0], 1.0 + g2 * g2, rtol=1e-9) and acc[1] == 0.25
    assert np.allclose(th[0], 1.9 - 0.1 * g2 / np.sqrt(1.0 + g2 * g2), rtol=1e-9)
    th, buf = np.array([2.0, 2.0]), np.zeros(2)
    O.sgd_update(th, np.array([0.5, 0.5]), buf, 1, 0.1, 0.9, 0.25, np.array([1.0, 0.0]))
    assert np.array_equal(buf, [1.0, 0.5]) and np.allclose(th, [1.9, 1.95], rtol=1e-15)
    O.sgd_update(th, np.array([0.25, 0.25]), buf, 2, 0.1, 0.9, 0.25, np.array([1.0, 0.0]))
    b0 = 0.9 * 1.0 + (0.25 + 0.25 * 1.9)        # = 1.625
    assert np.allclose(buf, [b0, 0.9 * 0.5 + 0.25], rtol=1e-15)
    assert np.allclose(th, [1.9 - 0.1 * b0, 1.95 - 0.07], rtol=1e-15)
    th = np.array([2.0])                         # no momentum: theta <- theta - lr (g + wd theta)
    O.sgd_update(th, np.array([0.5]), np.zeros(1), 1, 0.1, 0.0, 0.25, np.ones(1))
    assert np.allclose(th, 2.0 - 0.1 * 1.0, rtol=1e-15)


@pytest.mark.parametrize("kind", ["adagrad", "sgdm", "sgd"])
def test_adagrad_and_sgd_with_weight_decay_against_torch_optim(kind):
    """Three updates with a non-zero L2 decay against torch.optim's own implementations (float64)."""
    import torch
    rng = np.random.default_rng(3)
    n, lr, wd = 50, 0.05, 0.3
    th0 = rng.standard_normal(n)
    grads = [rng.standard_normal(n) for _ in range(3)]
    p = torch.nn.Parameter(torch.tensor(th0.copy()))
    if kind == "adagrad":
        topt = torch.optim.Adagrad([p], lr=lr, weight_decay=wd, eps=1e-10, initial_accumulator_value=0.0, lr_decay=0.0)
    else:
        topt = torch.optim.SGD([p], lr=lr, weight_decay=wd, momentum=0.9 if kind == "sgdm" else 0.0)
    th, st = th0.copy(), np.zeros(n)
    for t, g in enumerate(grads, 1):
        p.grad = torch.tensor(g.copy())
        topt.step()
        if kind == "adagrad":
            O.adagrad_update(th, g, st, lr, 1e-10, wd, np.ones(n))
        else:
            O.sgd_update(th, g, st, t, lr, 0.9 if kind == "sgdm" else 0.0, wd, np.ones(n))
        assert np.allclose(th, p.detach().numpy(), rtol=1e-13, atol=1e-15), (kind, t)


def test_per_group_step_counter_drives_bias_correction():
    # the second visit of a group is its update number 2, whatever the global step is
    o, _ = _fresh()
    k = o.set_group_schedule("bottom2up", 1, 0)
    for t in range(1, k + 2):
        tok, lab = make_batch(WL, 1, t)
        o.step(tok, lab, o.schedule_group_at(t))
    assert o.group_steps == [2, 1, 1, 1]


def test_delayed_learning_rate_changes_only_between_cycles():
    sgd = dict(kind="sgd", lr=1.0, beta1=0, beta2=0, eps=0, weight_decay=0.0, momentum=0.0)
    o, _ = _fresh(sgd)
    k = o.set_group_schedule("top2down", 1, 0)
    lrs = []
    for t in range(1, 3 * k + 1):
        lr = 1.0 / (1 + o.cycles_done)            # schedule indexed by completed cycles
        o.set_lr(lr)
        lrs.append(lr)
        tok, lab = make_batch(WL, 1, t)
        before = o.theta.copy()
        o.step(tok, lab, o.schedule_group_at(t))
        lo, hi = o.group_range(o.schedule_group_at(t))
        assert np.allclose((before - o.theta)[lo:hi], lr * o.last_grad[lo:hi], rtol=1e-10, atol=1e-15)
    assert lrs == [1.0] * k + [0.5] * k + [1 / 3] * k


def test_bf16_rounding_against_torch_conversion():
    import torch
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-6, 6, 20000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895313892515355e38, 1e-40]])
    ref = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float32).numpy().astype(np.float64)
    assert np.array_equal(O.bf16_round(x), ref)
    # ties go to the even neighbour: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert O.bf16_round(np.array([1.00390625]))[0] == 1.0
    assert O.bf16_round(np.array([1.01171875]))[0] == 1.015625


def test_half_weights_step_evaluates_at_rounded_master_and_updates_master():
    o, theta0 = _fresh()
    oh = O.HiftOracle(CFG, WL["opt"], theta0, half_weights=True)
    oh.set_group_schedule("bottom2up", 1, 0)
    tok, lab = make_batch(WL, 1, 1)
    loss = oh.step(tok, lab, 1)
    l_ref, g_ref = O.loss_and_grad(CFG, O.bf16_round(theta0), tok, lab)
    assert loss == l_ref and np.array_equal(oh.last_grad, g_ref)
    lo, hi = oh.group_range(1)
    p = WL["opt"]
    g = g_ref[lo:hi]
    exp = theta0[lo:hi] * (1 - p["lr"] * p["weight_decay"] * oh.decay_mask[lo:hi]) - p["lr"] * g / (np.abs(g) + p["eps"])
    assert np.allclose(oh.theta[lo:hi], exp, rtol=1e-12, atol=0)
    assert not np.array_equal(oh.theta[lo:hi], O.bf16_round(oh.theta[lo:hi]))   # master keeps full precision
    # later steps, too, are evaluated at the rounding of the master as it then is (the oracle keeps the rounded model
    # between steps and refreshes the group it updated: the same thing, written out here from scratch)
    for t in range(2, 7):
        gid = oh.schedule_group_at(t)
        tok, lab = make_batch(WL, 1, t)
        l_ref, g_ref = O.loss_and_grad(CFG, O.bf16_round(oh.theta), tok, lab)
        assert oh.step(tok, lab, gid) == l_ref and np.array_equal(oh.last_grad, g_ref), t


ADAFACTOR = dict(kind="adafactor", lr=1e-3, weight_decay=0.0)


def test_adafactor_first_step_by_hand():
    # one 1 x 2 matrix, G = [3, 4], first update (beta2_1 = 0): R = mean(9, 16) = 12.5, C = [9, 16],
    # V = R C / mean(R) = C, U = G / sqrt(C) = [1, 1], rms(U) = 1: not clipped
    th = np.array([0.5, -0.5])
    st = {}
    O.adafactor_update(th, np.array([3.0, 4.0]), st, (1, 2), 1, 0.1, 0.0, True)
    assert np.allclose(th, [0.4, -0.6], atol=1e-12)
    assert np.allclose(st["r"], [12.5]) and np.allclose(st["c"], [9.0, 16.0])
    # a vector with one large entry: U = sign(G) on the first step, so rms(U) = 1 again; with decay
    th = np.array([1.0, 1.0, 1.0])
    O.adafactor_update(th, np.array([2.0, -4.0, 8.0]), {}, (3,), 1, 0.1, 0.5, True)
    assert np.allclose(th, 1.0 - 0.1 * 0.5 - 0.1 * np.array([1.0, -1.0, 1.0]), atol=1e-12)
    # second step of a vector: beta2_2 = 1 - 2^-0.8; V = b V + (1 - b) G^2; |U| > 1 possible -> clipped to rms 1
    th, st = np.zeros(2), {}
    O.adafactor_update(th, np.array([1.0, 1.0]), st, (2,), 1, 1.0, 0.0, False)
    b = 1.0 - 2.0 ** -0.8
    g2 = np.array([3.0, 0.0])
    v = b * 1.0 + (1 - b) * (g2 * g2 + 1e-30)
    u = g2 / np.sqrt(v)
    u = u / max(1.0, np.sqrt(np.mean(u * u)))
    O.adafactor_update(th, g2, st, (2,), 2, 1.0, 0.0, False)
    assert np.allclose(th, -1.0 - u, atol=1e-12) and np.sqrt(np.mean(u * u)) <= 1.0 + 1e-12


def test_adafactor_against_the_transformers_implementation():
    """Same hyper-parameters (external step size, no parameter scaling, no momentum, clip 1.0,
    decay exponent 0.8, eps 1e-30): an independent implementation of the published algorithm."""
    import torch
    from transformers.optimization import Adafactor
    rng = np.random.default_rng(5)
    W0, b0 = rng.standard_normal((5, 7)), rng.standard_normal(6)
    W = torch.tensor(W0, dtype=torch.float64, requires_grad=True)
    b = torch.tensor(b0, dtype=torch.float64, requires_grad=True)
    opt = Adafactor([W, b], lr=0.01, relative_step=False, scale_parameter=False, warmup_init=False,
                    clip_threshold=1.0, decay_rate=-0.8, beta1=None, weight_decay=0.0, eps=(1e-30, 1e-3))
    thW, thb, sW, sb = W0.reshape(-1).copy(), b0.copy(), {}, {}
    for t in range(1, 5):
        gW, gb = rng.standard_normal((5, 7)) * (10.0 if t == 3 else 1.0), rng.standard_normal(6) * 0.01
        W.grad, b.grad = torch.tensor(gW), torch.tensor(gb)
        opt.step()
        O.adafactor_update(thW, gW.reshape(-1), sW, (5, 7), t, 0.01, 0.0, True)
        O.adafactor_update(thb, gb, sb, (6,), t, 0.01, 0.0, False)
        assert np.allclose(thW, W.detach().numpy().reshape(-1), rtol=1e-12, atol=1e-14)
        assert np.allclose(thb, b.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_adafactor_in_the_hift_loop_keeps_other_groups_frozen():
    o, _ = _fresh(ADAFACTOR)
    k = o.set_group_schedule("top2down", 1, 0)
    for t in range(1, 2 * k + 1):
        gid = o.schedule_group_at(t)
        before = o.theta.copy()
        tok, lab = make_batch(WL, 1, t)
        o.step(tok, lab, gid)
        lo, hi = o.group_range(gid)
        keep = np.ones(o.theta.size, bool)
        keep[lo:hi] = False
        assert np.array_equal(before[keep], o.theta[keep]) and not np.array_equal(before[lo:hi], o.theta[lo:hi])
    # factored state: n + m numbers for an n x m matrix, one per element for a vector
    total = sum(sum(v.size for v in st.values()) for st in o.factored.values())
    want = sum((s[0] + s[1]) if len(s) >= 2 else s[0] for _n, s, _k in SPEC)
    assert total == want


def test_cycle_indexed_linear_schedule_against_the_transformers_scheduler():
    """One scheduler step per sweep: the rate of cycle c is what the standard warm-up / linear-decay
    scheduler gives after c steps."""
    import torch
    from transformers import get_linear_schedule_with_warmup
    p = torch.nn.Parameter(torch.zeros(1))
    opt = torch.optim.SGD([p], lr=3e-5)
    sch = get_linear_schedule_with_warmup(opt, num_warmup_steps=3, num_training_steps=11)
    for c in range(13):
        assert abs(O.lr_at_cycle("linear", 3e-5, 3, 11, c) - sch.get_last_lr()[0]) <= 1e-18, c
        opt.step()
        sch.step()
    assert O.lr_at_cycle("constant", 0.1, 3, 11, 7) == 0.1
    assert O.lr_at_cycle("linear", 1.0, 0, 4, 0) == 1.0 and O.lr_at_cycle("linear", 1.0, 0, 4, 4) == 0.0


def test_rate_is_constant_inside_a_cycle_under_the_schedule():
    o, _ = _fresh(dict(kind="sgd", lr=0.0, momentum=0.0, weight_decay=0.0))
    k = o.set_group_schedule("bottom2up", 1, 0)
    seen = []
    for t in range(1, 3 * k + 1):
        o.set_lr(O.lr_at_cycle("linear", 1e-2, 1, 3, o.cycles_done))
        seen.append(o.opt["lr"])
        tok, lab = make_batch(WL, 1, t)
        o.step(tok, lab, o.schedule_group_at(t))
    assert all(len(set(seen[c * k:(c + 1) * k])) == 1 for c in range(3))
    assert seen[0] == 0.0 and seen[k] == 1e-2 and abs(seen[2 * k] - 0.5e-2) < 1e-18
