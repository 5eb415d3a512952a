"""GPU parity of the Adafactor update (factored second moments, update clipping) inside the HiFT
step, against the float64 oracle.  The update of element (i, j) is G_ij / sqrt(R_i C_j / mean R)
scaled by the clipping factor: its relative error is that of the gradient plus that of three
averages of squared gradients, so it is held to a small multiple of the gradient tolerance,
measured against |update| + rms of the tensor's update."""
import copy

import numpy as np
import pytest

from hift_inputs import WORKLOADS
from oracle import hift_oracle as O
from tests.hift_pair import make_pair, rel_l2, run_steps
from tests.test_gpu_step_fp32 import SMALL1, SMALL2

pytestmark = pytest.mark.gpu

ADAFACTOR = dict(kind="adafactor", lr=1e-3, weight_decay=0.01)


def _tensor_slices(orc, lo, hi):
    off = 0
    for i, (name, shape, _k, _u) in enumerate(O.param_tensors(orc.cfg)):
        n = int(np.prod(shape))
        if lo <= off and off + n <= hi:
            yield i, name, shape, off, n
        off += n


class Snapshot:
    """Oracle parameters, statistics and counters before a step."""

    def __init__(self, orc):
        self.theta = orc.theta.copy()
        self.factored = copy.deepcopy(orc.factored)
        self.steps = list(orc.group_steps)


def _check_update(orc, snap, gpu, gid, tb_g, ta_g, tol, outliers):
    """The allowed error of an element is the change of the oracle's own update when the tensor's
    gradient moves by tol * (|g| + rms g) (an element whose gradient is noise gets +-lr from a
    normalising optimizer on either side), plus 2 tol |update|, plus fp32 storage of theta."""
    lo, hi = orc.group_range(gid)
    frozen = np.ones(ta_g.size, bool)
    frozen[lo:hi] = False
    assert np.array_equal(tb_g[frozen], ta_g[frozen]), "frozen parameters changed"
    o, tg = orc.opt, snap.steps[gid] + 1
    for i, name, shape, off, n in _tensor_slices(orc, lo, hi):
        sl = slice(off, off + n)
        up_g = ta_g[sl].astype(np.float64) - tb_g[sl].astype(np.float64)
        up_o = orc.theta[sl] - snap.theta[sl]
        g = orc.last_grad[sl]
        delta = tol * (np.abs(g) + np.sqrt(np.mean(g * g)))
        slack = np.zeros(n)
        for sg in (+1.0, -1.0):
            th = snap.theta[sl].copy()
            O.adafactor_update(th, g + sg * delta, copy.deepcopy(snap.factored.get(name, {})), shape, tg, o["lr"],
                               o["weight_decay"], len(shape) >= 2)
            slack = np.maximum(slack, np.abs((th - snap.theta[sl]) - up_o))
        bound = 1.5 * slack + 2 * tol * np.abs(up_o) + 1.2e-7 * np.abs(snap.theta[sl])
        frac = float(np.mean(np.abs(up_g - up_o) > bound))
        assert frac <= outliers, (gid, name, frac, float(np.max(np.abs(up_g - up_o))))
        # the statistics themselves (averages of squared gradients: twice the gradient tolerance)
        st = orc.factored[name]
        ref = np.concatenate([st["r"], st["c"]]) if len(shape) >= 2 else st["v"]
        got = gpu.read_factored_state(i)
        assert rel_l2(got, ref) <= 4 * tol, (gid, name, rel_l2(got, ref))


@pytest.mark.parametrize("wl", [WORKLOADS["C1"], SMALL1, SMALL2], ids=["C1", "enc", "rope"])
def test_two_cycles_fp32(wl):
    orc, gpu, _ = make_pair(wl, seed=7, opt=ADAFACTOR, jitter=0.02)
    assert gpu.memory()["pinned_total"] == 0          # nothing to park on the host
    it = run_steps(orc, gpu, wl, 7, 2 * orc.k)
    while True:
        snap = Snapshot(orc)
        try:
            t, gid, lo_, lg, _chk, tb_g = next(it)
        except StopIteration:
            break
        assert abs(lg - lo_) <= 1e-5 * abs(lo_), (t, lo_, lg)
        _check_update(orc, snap, gpu, gid, tb_g, gpu.read_params(), 1e-5 if t <= orc.k else 4e-5, 0.0)


def test_state_on_host_flag_moves_nothing():
    orc, gpu, _ = make_pair(SMALL2, seed=8, opt=ADAFACTOR, state_on_host=1)
    it = run_steps(orc, gpu, SMALL2, 8, orc.k)
    for _ in it:
        pass
    assert gpu.transfer_stats() == (0, 0)


SMALL_ROPE_BF16 = dict(arch=2, n_layers=2, d_model=256, n_heads=4, d_ffn=512, vocab=1000, max_seq=128, n_classes=0,
                       norm_eps=1e-5, rope_base=10000.0, dtype=1, batch=2, seq=128, m=2, strategy="top2down", opt=None)


def test_two_cycles_bf16():
    orc, gpu, _ = make_pair(SMALL_ROPE_BF16, seed=9, opt=ADAFACTOR)
    it = run_steps(orc, gpu, SMALL_ROPE_BF16, 9, 2 * orc.k)
    while True:
        snap = Snapshot(orc)
        try:
            t, gid, lo_, lg, _chk, tb_g = next(it)
        except StopIteration:
            break
        assert abs(lg - lo_) <= 2e-2 * abs(lo_)
        _check_update(orc, snap, gpu, gid, tb_g, gpu.read_params(), 2e-2, 1e-3)


def test_7b_width_layer_group_bf16():
    # one update of a LLaMA-7B-width layer (matrices up to 22016 x 4096)
    wl = WORKLOADS["C4_L2"]
    orc, gpu, _ = make_pair(wl, seed=10, opt=ADAFACTOR)
    from hift_inputs import make_batch
    from tests.hift_pair import to_dev
    tok, lab = make_batch(wl, 10, 1)
    for gid in (1,):            # (the head's 32000 x 4096 matrix goes through the same kernels; its group is covered at the small shapes)
        snap = Snapshot(orc)
        tb_g = gpu.read_params()
        lo_ = orc.step(tok, lab, gid)
        lg = gpu.step(*to_dev(tok, lab), gid)
        assert abs(lg - lo_) <= 2e-2 * abs(lo_)
        # 2048-token sums: a few more elements than at the small shape land where the terms nearly cancel
        _check_update(orc, snap, gpu, gid, tb_g, gpu.read_params(), 2e-2, 2e-3)
