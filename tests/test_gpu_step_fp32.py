"""GPU parity, fp32 mode: the HIP path against the float64 oracle on the tiny decoder (C1) and on
small fp32 instances of the other two architectures.  Tolerance 1e-5 relative on the loss and on
the update of the active group; frozen parameters bit-identical; schedules bit-exact."""
import numpy as np
import pytest

from hift_inputs import WORKLOADS, make_batch
from oracle import hift_oracle as O
from tests.hift_pair import make_pair, rel_l2, run_steps, to_dev

pytestmark = pytest.mark.gpu

TOL = 1e-5

SMALL1 = dict(arch=1, n_layers=2, d_model=64, n_heads=4, d_ffn=128, vocab=300, max_seq=40, n_classes=3,
              norm_eps=1e-5, rope_base=10000.0, dtype=0, batch=4, seq=24, m=1, strategy="top2down",
              opt=WORKLOADS["C1"]["opt"])
SMALL2 = dict(arch=2, n_layers=2, d_model=64, n_heads=4, d_ffn=96, vocab=320, max_seq=48, n_classes=0,
              norm_eps=1e-5, rope_base=10000.0, dtype=0, batch=2, seq=40, m=1, strategy="random",
              opt=WORKLOADS["C1"]["opt"])
# GPT-2 / OPT style: the output matrix is the token table (section 4.1 lists both families)
TIED0 = dict(WORKLOADS["C1"], tie_embeddings=1)
TIED2 = dict(SMALL2, tie_embeddings=1)
SGD1 = dict(kind="sgd", lr=1.0, beta1=0, beta2=0, eps=0, weight_decay=0.0, momentum=0.0)


@pytest.mark.parametrize("wl", [WORKLOADS["C1"], SMALL1, SMALL2, TIED0, TIED2], ids=["C1", "enc", "rope", "C1_tied", "rope_tied"])
def test_two_cycles_adamw(wl):
    orc, gpu, _ = make_pair(wl, seed=3, jitter=0.02)
    k = orc.k
    for t, gid, lo_, lg, chk, tb_g in run_steps(orc, gpu, wl, 3, 2 * k):
        assert abs(lg - lo_) <= TOL * abs(lo_), (t, lo_, lg)
        ta_g = gpu.read_params()
        lo, hi = orc.group_range(gid)
        frozen = np.ones(ta_g.size, bool)
        frozen[lo:hi] = False
        assert np.array_equal(tb_g[frozen], ta_g[frozen]), "frozen parameters changed"
        # first sweep: the update itself to TOL; later sweeps start from parameters and state
        # that already differ by fp32 rounding, so the update is held to 4 TOL there
        ok, info = chk.check(tb_g, ta_g, TOL if t <= k else 4 * TOL)
        assert ok, (t, gid, info)
        assert rel_l2(ta_g[lo:hi], orc.theta[lo:hi]) <= TOL
    assert gpu.cycle_index() == (2 * k, 2)


@pytest.mark.parametrize("wl", [WORKLOADS["C1"], SMALL1, SMALL2, TIED0, TIED2], ids=["C1", "enc", "rope", "C1_tied", "rope_tied"])
def test_gradient_of_every_group_via_sgd(wl):
    # SGD, lr 1, no momentum/decay: theta0 - theta1 is the gradient of the active group
    tok, lab = make_batch(wl, 5, 1)
    dtok, dlab = to_dev(tok, lab)
    orc, gpu, theta0 = make_pair(wl, seed=5, opt=SGD1, jitter=0.02)
    _l, g = O.loss_and_grad(orc.cfg, theta0.astype(np.float64), tok, lab)
    for gid in range(orc.k):
        gpu.write_params(0, gpu.n_units, theta0)
        gpu.step(dtok, dlab, gid)
        lo, hi = orc.group_range(gid)
        got = (theta0.astype(np.float64) - gpu.read_params().astype(np.float64))[lo:hi]
        ref = g[lo:hi]
        assert rel_l2(got, ref) <= 3 * TOL, (gid, rel_l2(got, ref))
        assert np.max(np.abs(got - ref)) <= 3 * TOL * np.max(np.abs(ref)) + 1.2e-7 * np.max(np.abs(theta0[lo:hi]))


@pytest.mark.parametrize("optk", ["adagrad", "sgdm"])
def test_other_optimizers(optk):
    wl = WORKLOADS["C1"]
    opt = (dict(kind="adagrad", lr=1e-2, eps=1e-10, weight_decay=0.0) if optk == "adagrad"
           else dict(kind="sgd", lr=1e-2, momentum=0.9, weight_decay=0.0))
    orc, gpu, _ = make_pair(wl, seed=9, opt=opt, jitter=0.02)
    for t, gid, lo_, lg, chk, tb_g in run_steps(orc, gpu, wl, 9, 2 * orc.k):
        assert abs(lg - lo_) <= TOL * abs(lo_)
        ok, info = chk.check(tb_g, gpu.read_params(), TOL if t <= orc.k else 4 * TOL)
        assert ok, (t, gid, info)


def test_single_group_is_full_finetuning_step():
    wl = WORKLOADS["C1"]
    orc, gpu, _ = make_pair(wl, seed=2, m=4, jitter=0.02)
    assert orc.k == 1 and gpu.k == 1
    for t, gid, lo_, lg, chk, tb_g in run_steps(orc, gpu, wl, 2, 3):
        assert abs(lg - lo_) <= TOL * abs(lo_)
    assert rel_l2(gpu.read_params(), orc.theta) <= TOL


@pytest.mark.parametrize("engine", [0, 1], ids=["memcpy_async", "copy_kernel"])
def test_state_offload_matches_resident_state_bitwise(engine):
    wl = WORKLOADS["C1"]
    _o1, g_res, _ = make_pair(wl, seed=4, state_on_host=0, jitter=0.02)
    _o2, g_off, _ = make_pair(wl, seed=4, state_on_host=1, jitter=0.02)
    g_off.set_state_copy_engine(engine, 4)
    k = g_res.k
    for t in range(1, 3 * k + 1):
        gid = g_res.schedule_group_at(t)
        tok, lab = make_batch(wl, 4, t)
        dtok, dlab = to_dev(tok, lab)
        l1 = g_res.step(dtok, dlab, gid)
        l2 = g_off.step(dtok, dlab, gid)
        assert l1 == l2
    assert np.array_equal(g_res.read_params(), g_off.read_params())
    for slot in (0, 1):
        assert np.array_equal(g_res.read_state(0, g_res.n_units, slot), g_off.read_state(0, g_off.n_units, slot))
    h2d, d2h = g_off.transfer_stats()
    assert d2h == 3 * 2 * 4 * g_off.n_params and h2d >= d2h      # every group written back once per cycle
    assert g_res.transfer_stats() == (0, 0)


def test_off_schedule_group_takes_the_synchronous_fetch_and_stays_correct():
    wl = WORKLOADS["C1"]
    orc, gpu, _ = make_pair(wl, seed=6, state_on_host=1, jitter=0.02)
    seq = [2, 2, 0, 3, 1, 1, 0]
    for t, gid in enumerate(seq, 1):
        tok, lab = make_batch(wl, 6, t)
        dtok, dlab = to_dev(tok, lab)
        lo_ = orc.step(tok, lab, gid)
        lg = gpu.step(dtok, dlab, gid)
        assert abs(lg - lo_) <= TOL * abs(lo_)
    assert rel_l2(gpu.read_params(), orc.theta) <= TOL


@pytest.mark.parametrize("bf16", [0, 1])
def test_one_token_sequences_have_no_target(bf16):
    """Sequences of one token give the decoder nothing to predict: loss 0, no gradient; AdamW then only decays the
    matrices of the active group, as in the oracle."""
    wl = dict(SMALL2, dtype=1) if bf16 else WORKLOADS["C1"]
    orc, gpu, _ = make_pair(wl, seed=2)
    tok, lab = make_batch(wl, 2, 1, batch=2, seq=1)
    assert (lab < 0).all()
    for t in range(1, orc.k + 1):
        gid = orc.schedule_group_at(t)
        lo_ = orc.step(tok, lab, gid)
        lg = gpu.step(*to_dev(tok, lab), gid)
        assert lo_ == 0.0 and lg == 0.0
    got = gpu.read_params().astype(np.float64)
    assert np.isfinite(got).all()
    assert rel_l2(got, orc.theta) <= TOL


def test_plain_sgd_moves_no_state():
    wl = WORKLOADS["C1"]
    orc, gpu, _ = make_pair(wl, seed=7, opt=dict(kind="sgd", lr=0.1, momentum=0.0, weight_decay=0.0), state_on_host=1)
    for _ in run_steps(orc, gpu, wl, 7, orc.k):
        pass
    assert gpu.transfer_stats() == (0, 0) and gpu.pinned_bytes == 0


def test_schedule_and_layout_bit_exact():
    import paper_2401_15207_amd as H
    for name in ("C1", "C2", "C3", "C4", "C5"):
        wl = WORKLOADS[name]
        from hift_inputs import model_config
        cfg = model_config(wl)
        tl, n = H.tensor_list(cfg)
        ref = O.param_tensors(cfg)
        assert n == O.n_params(cfg) and len(tl) == len(ref)
        off = 0
        for (gn, gs, gk, gu, go), (rn, rs, rk, ru) in zip(tl, ref):
            assert (gn, tuple(gs), gk, gu, go) == (rn, tuple(rs), rk, ru, off)
            off += int(np.prod(rs))
        n_units = wl["n_layers"] + 2
        for m in (1, 2, 3, 4, n_units):
            k = H.group_count(n_units, m)
            assert k == O.n_groups(n_units, m)
            for s in ("bottom2up", "top2down", "random"):
                assert H.group_order(k, s, 123) == O.group_order(k, s, 123)


def test_error_paths():
    import paper_2401_15207_amd as H
    wl = WORKLOADS["C1"]
    orc, gpu, _ = make_pair(wl, seed=1)
    tok, lab = make_batch(wl, 1, 1)
    dtok, dlab = to_dev(tok, lab)
    with pytest.raises(H.HiftError):
        gpu.step(dtok, dlab, 4)
    with pytest.raises(H.HiftError):
        gpu.step(dtok, dlab, -1)
    big_tok, big_lab = to_dev(np.zeros((3, 32), np.int32), np.zeros((3, 32), np.int32))
    with pytest.raises(H.HiftError):
        gpu.step(big_tok, big_lab, 0)
    with pytest.raises(H.HiftError):
        gpu.set_group_schedule("bottom2up", 0)
    with pytest.raises(H.HiftError):
        gpu.read_params(2, 1)
    # ragged batch below the maxima is fine
    tok, lab = make_batch(wl, 1, 2, batch=1, seq=17)
    dtok, dlab = to_dev(tok, lab)
    lo_ = orc.step(tok, lab, 1)
    lg = gpu.step(dtok, dlab, 1)
    assert abs(lg - lo_) <= TOL * abs(lo_)


@pytest.mark.parametrize("optk", ["adamw", "sgdm"])
def test_regrouping_keeps_state_and_update_counts(optk):
    """Setting a schedule again keeps the optimizer state and each unit's update count: a run that regroups between
    two updates of the same units (one unit per group -> two units per group) ends bit-identical, on those units,
    to a run that updates them one by one the second time as well.  (Were the count reset, SGD with momentum would
    overwrite its buffer with the raw gradient and AdamW would restart its bias correction on non-zero moments.)"""
    wl = WORKLOADS["C1"]
    opt = (wl["opt"] if optk == "adamw" else dict(kind="sgd", lr=1e-2, momentum=0.9, weight_decay=0.0))
    _o, a, _t = make_pair(wl, seed=7, opt=opt, m=1, strategy="bottom2up", state_on_host=1)
    _o, b, _t = make_pair(wl, seed=7, opt=opt, m=2, strategy="bottom2up", state_on_host=1)   # buffers sized for two units
    batches = [to_dev(*make_batch(wl, 7, t)) for t in (1, 2, 3)]
    for mdl in (a, b):
        assert mdl.set_group_schedule("bottom2up", 1, 0) == 4
        mdl.step(*batches[0], 1)             # layer 0 and layer 1, once each
        mdl.step(*batches[1], 2)
    # a: layer 0 again on its own.  b: regroup to {emb, layer 0}, {layer 1, head} and update the first group
    a.step(*batches[2], 1)
    assert b.set_group_schedule("bottom2up", 2, 0) == 2
    b.step(*batches[2], 0)
    assert np.array_equal(a.read_params(1, 2), b.read_params(1, 2))
    for j in range(2 if optk == "adamw" else 1):
        assert np.array_equal(a.read_state(1, 2, j), b.read_state(1, 2, j))


@pytest.mark.parametrize("master_on_host", [0, 1])
def test_pinned_arena_in_chunks_changes_nothing(master_on_host):
    """The pinned arena handed in as many small blocks (here 4112 bytes each, so that the state of every group
    straddles several of them) against one block: losses, parameters, state and checkpoints bit-identical."""
    import paper_2401_15207_amd as H
    wl = dict(SMALL2, dtype=1) if master_on_host else WORKLOADS["C1"]
    cfg = {k: wl[k] for k in ("arch", "n_layers", "d_model", "n_heads", "d_ffn", "vocab", "max_seq", "n_classes",
                              "norm_eps", "rope_base", "dtype")}
    spec = [(n, s, k) for n, s, k, _u in O.param_tensors(cfg)]
    from hift_inputs import init_params
    theta0 = init_params(9, spec, bf16_exact=bool(cfg["dtype"]))
    models = [H.HiftModel(cfg, wl["opt"], 1, wl["batch"], wl["seq"], init_params=theta0, state_on_host=1,
                          master_on_host=master_on_host, pinned_chunk_bytes=cb) for cb in (1 << 40, 4112)]
    assert len(models[0].pinned_chunks) == 1 and len(models[1].pinned_chunks) > 20
    for mdl in models:
        assert mdl.set_group_schedule("random", 1, 3) == 4
    for t in range(1, 9):
        batch = to_dev(*make_batch(wl, 9, t))
        gid = models[0].schedule_group_at(t)
        la, lb = (mdl.step(*batch, gid) for mdl in models)
        assert la == lb, t
    a, b = models
    assert np.array_equal(a.read_params(), b.read_params())
    assert np.array_equal(a.read_params(which=1), b.read_params(which=1))
    for j in (0, 1):
        assert np.array_equal(a.read_state(0, a.n_units, j), b.read_state(0, b.n_units, j))
    ck = b.checkpoint_save()
    assert np.array_equal(ck, a.checkpoint_save())
    b.write_params(1, 2, theta0[:0].tolist() + list(a.read_params(1, 2) * 0))    # disturb, then restore from the checkpoint
    b.checkpoint_load(ck)
    assert np.array_equal(a.read_params(), b.read_params())
    batch = to_dev(*make_batch(wl, 9, 9))
    assert a.step(*batch, 2) == b.step(*batch, 2)
    assert np.array_equal(a.read_params(), b.read_params())


@pytest.mark.parametrize("bf16,master_on_host", [(0, 0), (1, 0), (1, 1)])
def test_parameters_written_from_device_memory(bf16, master_on_host):
    # hift_write_params_device: the same parameters, forward copy and (through a step) packed copies as the host writer
    import torch
    wl = dict(SMALL2, dtype=bf16)
    _o, a, theta0 = make_pair(wl, seed=14, state_on_host=1, master_on_host=master_on_host)
    _o, b, _t = make_pair(wl, seed=15, state_on_host=1, master_on_host=master_on_host)     # other weights
    off = 0
    for u in range(b.n_units):
        n = b._unit_count(u, u + 1)
        b.write_params_device(u, u + 1, torch.from_numpy(theta0[off:off + n].copy()).cuda())
        off += n
    assert np.array_equal(a.read_params(), b.read_params()) and np.array_equal(a.read_params(which=1), b.read_params(which=1))
    batch = to_dev(*make_batch(wl, 14, 1))
    gid = a.schedule_group_at(1)
    assert a.step(*batch, gid) == b.step(*batch, gid)
    assert np.array_equal(a.read_params(), b.read_params())
