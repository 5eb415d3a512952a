"""GPU parity, bf16 mode (bf16 weights and activations, fp32 accumulation, fp32 master weights)
against the float64 oracle.  Both sides start from bf16-representable weights.  Tolerance 2e-2
relative on the loss and on gradients / updates of the active group (L2 over the group and per
element against the tensor's scale); frozen parameters, group indexing and schedules bit-exact."""
import numpy as np
import pytest

from hift_inputs import WORKLOADS, init_params, make_batch, model_config, round_to_bf16
from oracle import hift_oracle as O
from tests.hift_pair import make_pair, rel_l2, run_steps, spec_of, to_dev

pytestmark = pytest.mark.gpu

TOL = 2e-2
SGD1 = dict(kind="sgd", lr=1.0, beta1=0, beta2=0, eps=0, weight_decay=0.0, momentum=0.0)


def _depth_tol(orc, ulo):
    """Gradient tolerance of a group whose lowest unit is ulo.  Every bf16 rounding on the way
    from the loss down to the group adds an independent relative error of about 2^-9/sqrt(3);
    a layer has about 25 of them, so the error grows with the square root of the number of
    layers the backward pass crosses.  2e-2 covers four layers; deeper groups get
    2e-2 * sqrt(layers / 4)."""
    layers = orc.cfg["n_layers"] - max(ulo, 1) + 1
    return TOL * max(1.0, np.sqrt(layers / 4.0))


def _check_group_gradient(orc, got, ref, lo, hi, label, TOL=TOL):
    """got / ref: flat gradients of one group.  The criterion proper is the relative L2 error:
    TOL over the group, 1.5 TOL per tensor (TOL = 2e-2 scaled for depth, see _depth_tol).  To catch errors confined to a few rows, which an L2
    over a large tensor would hide, 99.9 % of the elements of every tensor must also lie within
    5 TOL of (|ref| + rms of the tensor's non-zero reference gradient)."""
    assert rel_l2(got, ref) <= TOL, (label, rel_l2(got, ref))
    off = 0
    for name, shape, _k, _u in O.param_tensors(orc.cfg):
        n = int(np.prod(shape))
        a, b = max(off, lo), min(off + n, hi)
        if a < b:
            r, g = ref[a - lo:b - lo], got[a - lo:b - lo]
            nz = r != 0
            rms = np.sqrt(np.mean(r[nz] ** 2)) if nz.any() else 0.0
            if rms > 0 and not name.endswith("bqkv"):   # the key-bias third has an identically zero gradient
                frac = np.mean(np.abs(g - r) > 5 * TOL * (np.abs(r) + rms))
                assert frac <= 1e-3, (label, name, float(frac))
                assert rel_l2(g, r) <= 1.5 * TOL, (label, name, rel_l2(g, r))
        off += n


def _gradient_check(wl, groups, seed=5, **over):
    tok, lab = make_batch(wl, seed, 1)
    dtok, dlab = to_dev(tok, lab)
    orc, gpu, theta0 = make_pair(wl, seed=seed, opt=SGD1, **over)
    lo_, g = O.loss_and_grad(orc.cfg, theta0.astype(np.float64), tok, lab)
    for gid in groups(orc.k):
        ulo, uhi = gpu.group_units(gid)
        lo, hi = orc.group_range(gid)
        lg = gpu.step(dtok, dlab, gid)
        assert abs(lg - lo_) <= TOL * abs(lo_), (lg, lo_)
        after = gpu.read_params(ulo, uhi).astype(np.float64)
        got = theta0[lo:hi].astype(np.float64) - after
        _check_group_gradient(orc, got, g[lo:hi], lo, hi, f"group {gid}", _depth_tol(orc, ulo))
        # the forward copy of the group is the rounded master; put the start values back
        fw = gpu.read_params(ulo, uhi, which=1)
        assert np.array_equal(fw, round_to_bf16(after.astype(np.float32)))
        gpu.write_params(ulo, uhi, theta0[lo:hi])
    return orc, gpu


def test_c2_full_shape_gradients_of_sampled_groups():
    # RoBERTa-base shape at its full size; groups: embeddings, a middle layer, top layer, head
    _gradient_check(WORKLOADS["C2"], lambda k: [0, 6, k - 2, k - 1])


def test_c3_shape_reduced_depth_random_schedule_adamw():
    wl = dict(WORKLOADS["C3"], n_layers=4)
    orc, gpu, _ = make_pair(wl, seed=8, sched_seed=99)
    assert orc.k == 3 and orc.order == gpu_order(gpu)
    for t, gid, lo_, lg, chk, tb_g in run_steps(orc, gpu, wl, 8, 2 * orc.k):
        assert abs(lg - lo_) <= TOL * abs(lo_), (t, lo_, lg)
        ta_g = gpu.read_params()
        lo, hi = orc.group_range(gid)
        frozen = np.ones(ta_g.size, bool)
        frozen[lo:hi] = False
        assert np.array_equal(tb_g[frozen], ta_g[frozen])
        ok, info = chk.check(tb_g, ta_g, TOL, max_outlier_frac=1e-3)
        assert ok, (t, gid, info)


def gpu_order(gpu):
    return [gpu.schedule_group_at(t) for t in range(1, gpu.k + 1)]


def test_c2_reduced_depth_top2down_adamw_with_offload():
    wl = dict(WORKLOADS["C2"], n_layers=3)
    orc, gpu, _ = make_pair(wl, seed=4, state_on_host=1)
    assert gpu_order(gpu) == [4, 3, 2, 1, 0]
    for t, gid, lo_, lg, chk, tb_g in run_steps(orc, gpu, wl, 4, 2 * orc.k):
        assert abs(lg - lo_) <= TOL * abs(lo_), (t, lo_, lg)
        ok, info = chk.check(tb_g, gpu.read_params(), TOL, max_outlier_frac=1e-3)
        assert ok, (t, gid, info)
    # optimizer state of every unit came back to the host; AdamW first moment ~ oracle's
    m_g = gpu.read_state(0, gpu.n_units, 0)
    assert rel_l2(m_g, orc.state1) <= 2 * TOL


def test_c4_width_two_layers_gradients_all_groups():
    # LLaMA-7B widths (d 4096, 32 heads, SwiGLU 11008, vocab 32000), batch 4 x 512, depth 2
    _gradient_check(WORKLOADS["C4_L2"], lambda k: range(k))


def test_tied_embeddings_on_the_packed_kernels():
    # The token table doubles as output matrix (GPT-2 / OPT style) and is wide enough to get fragment-order
    # copies: forward head, head dX and the two-part gradient of the table all run on the fast kernels.
    wl = dict(arch=2, n_layers=2, d_model=1024, n_heads=8, d_ffn=2816, vocab=8192, max_seq=512, n_classes=0,
              norm_eps=1e-5, rope_base=10000.0, dtype=1, batch=4, seq=512, m=1, strategy="bottom2up",
              opt=WORKLOADS["C4"]["opt"], tie_embeddings=1)
    orc, gpu = _gradient_check(wl, lambda k: range(k))
    assert gpu.n_units == 4 and [n for n, *_ in gpu.tensors][-1] == "gf"      # no separate output matrix


def test_c5_width_two_layers_group_of_two_units():
    wl = dict(WORKLOADS["C5_L2"], batch=1)
    _gradient_check(wl, lambda k: [1], m=2)


@pytest.mark.parametrize("optk", ["adagrad", "sgdm"])
def test_small_rope_decoder_other_optimizers_bf16(optk):
    wl = dict(arch=2, n_layers=2, d_model=256, n_heads=4, d_ffn=512, vocab=1000, max_seq=128, n_classes=0,
              norm_eps=1e-5, rope_base=10000.0, dtype=1, batch=2, seq=128, m=2, strategy="top2down", opt=None)
    opt = (dict(kind="adagrad", lr=1e-3, eps=1e-10, weight_decay=0.0) if optk == "adagrad"
           else dict(kind="sgd", lr=1e-2, momentum=0.9, weight_decay=0.0))
    orc, gpu, _ = make_pair(wl, seed=12, opt=opt, state_on_host=1)
    for t, gid, lo_, lg, chk, tb_g in run_steps(orc, gpu, wl, 12, 2 * orc.k):
        assert abs(lg - lo_) <= TOL * abs(lo_)
        ok, info = chk.check(tb_g, gpu.read_params(), TOL, max_outlier_frac=1e-3)
        assert ok, (t, gid, info)


SMALL_ROPE = dict(arch=2, n_layers=3, d_model=256, n_heads=4, d_ffn=512, vocab=1000, max_seq=128, n_classes=0,
                  norm_eps=1e-5, rope_base=10000.0, dtype=1, batch=2, seq=128, m=1, strategy="random", opt=None)


@pytest.mark.parametrize("optk", ["adamw", "sgd"])
def test_master_on_host_gives_the_same_trajectory(optk):
    """Adapted mixed precision (appendix "Mixing Precision"): with the fp32 master of the inactive groups
    parked on the host, every step must produce bit-identical weights, state and loss to the run that
    keeps the master in HBM, and stay within tolerance of the oracle."""
    opt = (dict(kind="adamw", lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01) if optk == "adamw"
           else dict(kind="sgd", lr=1e-2, momentum=0.0, weight_decay=0.0))
    orc, hbm, theta0 = make_pair(SMALL_ROPE, seed=21, opt=opt, state_on_host=1)
    _o, host, _t = make_pair(SMALL_ROPE, seed=21, opt=opt, state_on_host=1, master_on_host=1)
    assert np.array_equal(host.read_params(), theta0) and np.array_equal(host.read_params(which=1), hbm.read_params(which=1))
    for t, gid, lo_, lg, chk, tb_g in run_steps(orc, hbm, SMALL_ROPE, 21, 2 * orc.k):
        tok, lab = make_batch(SMALL_ROPE, 21, t)
        lh = host.step(*to_dev(tok, lab), gid)
        assert lh == lg, (t, lh, lg)
        after = hbm.read_params()
        assert np.array_equal(host.read_params(), after), t
        assert np.array_equal(host.read_params(which=1), hbm.read_params(which=1)), t
        assert abs(lg - lo_) <= TOL * abs(lo_)
        ok, info = chk.check(tb_g, after, TOL, max_outlier_frac=1e-3)
        assert ok, (t, gid, info)
    if optk == "adamw":
        for j in (0, 1):
            assert np.array_equal(host.read_state(0, host.n_units, j), hbm.read_state(0, hbm.n_units, j))
    # writing parameters goes to the host master and refreshes the forward copy
    ulo, uhi = host.group_units(1)
    lo, hi = orc.group_range(1)
    host.write_params(ulo, uhi, theta0[lo:hi])
    hbm.write_params(ulo, uhi, theta0[lo:hi])
    assert np.array_equal(host.read_params(), hbm.read_params())
    tok, lab = make_batch(SMALL_ROPE, 21, 99)
    assert host.step(*to_dev(tok, lab), 1) == hbm.step(*to_dev(tok, lab), 1)
    assert np.array_equal(host.read_params(), hbm.read_params())
    m = host.memory()
    assert m["device_master"] < hbm.memory()["device_master"]


def test_c4_width_without_packed_copies():
    # the contractions read the row-major bf16 copy when the fragment-order copies are switched off
    _gradient_check(WORKLOADS["C4_L2"], lambda k: [1, k - 1], no_packed_copies=1)
