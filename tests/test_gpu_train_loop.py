"""GPU tests of the multi-step entry points: the train loop with the cycle-indexed learning-rate
schedule (delayed update, section 3) against the oracle run step by step, and checkpoint / resume."""
import numpy as np
import pytest

from hift_inputs import make_batch
from oracle import hift_oracle as O
from tests.hift_pair import make_pair, rel_l2, to_dev
from tests.test_gpu_step_fp32 import SMALL2

pytestmark = pytest.mark.gpu

TOL = 1e-5


def _batches(wl, seed, n):
    host = [make_batch(wl, seed, t) for t in range(1, n + 1)]
    return host, [to_dev(tok, lab) for tok, lab in host]


@pytest.mark.parametrize("optk", ["adamw", "sgd"])
def test_train_loop_with_linear_schedule_follows_the_oracle(optk):
    opt = (dict(kind="adamw", lr=0.0, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01) if optk == "adamw"
           else dict(kind="sgd", lr=0.0, momentum=0.9, weight_decay=0.0))
    orc, gpu, _ = make_pair(SMALL2, seed=31, opt=opt, strategy="bottom2up", jitter=0.02, state_on_host=1)
    k = orc.k
    base, warm, total = (2e-3 if optk == "adamw" else 5e-2), 1, 4
    host, dev = _batches(SMALL2, 31, 5)
    gpu.set_lr_schedule("linear", base, warm, total)
    n = 3 * k + 2
    losses = gpu.train(dev, n)
    ref = []
    for i in range(n):
        lr = O.lr_at_cycle("linear", base, warm, total, orc.cycles_done)
        assert lr == pytest.approx(__import__("paper_2401_15207_amd").lr_at_cycle("linear", base, warm, total, orc.cycles_done), abs=0)
        orc.set_lr(lr)
        tok, lab = host[i % 5]
        ref.append(orc.step(tok, lab, orc.schedule_group_at(i + 1)))
    assert np.allclose(losses, ref, rtol=4 * TOL, atol=0)
    assert gpu.cycle_index() == (n, 3)
    # the first sweep runs at rate 0 (warm-up of one cycle): nothing may have moved before it ends;
    # afterwards the trajectory follows the oracle's
    assert rel_l2(gpu.read_params(), orc.theta) <= 8 * TOL
    # without losses the loop never waits for the GPU; same result
    orc2, gpu2, _ = make_pair(SMALL2, seed=31, opt=opt, strategy="bottom2up", jitter=0.02, state_on_host=1)
    gpu2.set_lr_schedule("linear", base, warm, total)
    assert gpu2.train(dev, n, want_losses=False) is None
    assert np.array_equal(gpu2.read_params(), gpu.read_params())   # no kernel sums in a timing-dependent order


def test_rate_zero_sweep_changes_nothing():
    opt = dict(kind="sgd", lr=1.0, momentum=0.0, weight_decay=0.0)
    orc, gpu, theta0 = make_pair(SMALL2, seed=32, opt=opt, strategy="random")
    _h, dev = _batches(SMALL2, 32, 3)
    gpu.set_lr_schedule("linear", 1.0, 2, 5)           # cycle 0 runs at 0
    gpu.train(dev, orc.k, want_losses=False)
    assert np.array_equal(gpu.read_params(), theta0)


@pytest.mark.parametrize("optk,on_host", [("adamw", 1), ("adamw", 0), ("adafactor", 0)])
def test_checkpoint_resume_continues_bit_identically(optk, on_host):
    opt = (dict(kind="adamw", lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01) if optk == "adamw"
           else dict(kind="adafactor", lr=1e-3, weight_decay=0.0))
    _o, a, theta0 = make_pair(SMALL2, seed=33, opt=opt, strategy="top2down", state_on_host=on_host)
    k = a.k                                             # top2down: head, layer 1, layer 0, embeddings
    _h, dev = _batches(SMALL2, 33, 4)
    a.set_lr_schedule("linear", 1e-3, 1, 6)
    a.train(dev, k + 1, want_losses=False)              # one sweep and the head again
    ckpt = a.checkpoint_save()
    la = a.train(dev, k + 1)                            # through the embeddings and round again
    _o, b, _t = make_pair(SMALL2, seed=34, opt=opt, strategy="bottom2up", state_on_host=on_host)   # other weights, other order
    b.checkpoint_load(ckpt)
    assert b.cycle_index() == (k + 1, 1) and [b.schedule_group_at(t) for t in range(1, k + 1)] == list(range(k - 1, -1, -1))
    lb = b.train(dev, k + 1)
    assert np.array_equal(la, lb)
    assert np.array_equal(a.read_params(), b.read_params())
    if optk == "adamw":
        for j in (0, 1):
            assert np.array_equal(a.read_state(0, a.n_units, j), b.read_state(0, b.n_units, j))
    else:
        for i in range(len(a.tensors)):
            assert np.array_equal(a.read_factored_state(i), b.read_factored_state(i))
    # a checkpoint of another optimizer or a damaged buffer is refused
    import paper_2401_15207_amd as H
    with pytest.raises(H.HiftError):
        b.checkpoint_load(ckpt[:100])
    bad = ckpt.copy()
    bad[:4] = 0
    with pytest.raises(H.HiftError):
        b.checkpoint_load(bad)
    # a checkpoint whose visiting order is damaged (a group twice) is refused before anything of the model changes
    pat = np.arange(k - 1, -1, -1, dtype=np.int32).view(np.uint8)
    at = next(i for i in range(256) if np.array_equal(ckpt[i:i + pat.size], pat))
    bad = ckpt.copy()
    bad[at:at + 4] = bad[at + 4:at + 8]
    bad[at + 4 * k + 200:at + 4 * k + 10000] = 0xFF     # and so are its parameters
    before = (b.cycle_index(), b.read_params(), [b.schedule_group_at(t) for t in range(1, k + 1)])
    with pytest.raises(H.HiftError):
        b.checkpoint_load(bad)
    assert b.cycle_index() == before[0] and np.array_equal(b.read_params(), before[1])
    assert [b.schedule_group_at(t) for t in range(1, k + 1)] == before[2]
    assert np.array_equal(b.train(dev, 2), a.train(dev, 2))   # and it goes on exactly as the run it mirrors


@pytest.mark.timeout(600)
@pytest.mark.parametrize("master_on_host", [0, 1])
def test_checkpoint_resume_at_the_7b_widths_in_bf16(master_on_host):
    """The same at the LLaMA-7B widths (depth 2), where the matrices exist in HBM only in fragment order (or, with the
    master on the host, as a bf16 copy besides): a model of other weights and another order takes the checkpoint
    and continues bit for bit: losses, master, compute copy, optimizer state."""
    import paper_2401_15207_amd as H
    from hift_inputs import WORKLOADS, init_params, model_config
    from tests.hift_pair import spec_of
    wl = WORKLOADS["C4_L2"]
    cfg = model_config(wl)
    opt = dict(kind="adamw", lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
    _h, dev = _batches(wl, 33, 4)

    theta = init_params(33, spec_of(cfg), bf16_exact=True)

    def model(values, strategy):
        m = H.HiftModel(cfg, opt, 1, wl["batch"], wl["seq"], init_params=values, state_on_host=1, master_on_host=master_on_host)
        m.set_group_schedule(strategy, 1, 17)
        return m

    a = model(theta, "top2down")
    k = a.k
    a.set_lr_schedule("linear", 1e-4, 1, 6)
    a.train(dev, k + 1, want_losses=False)
    ckpt = a.checkpoint_save()
    la = a.train(dev, k + 1)
    b = model(np.ascontiguousarray(theta[::-1]), "bottom2up")     # other weights (the same values in reverse), other order
    del theta
    b.checkpoint_load(ckpt)
    del ckpt
    lb = b.train(dev, k + 1)
    assert np.isfinite(la).all() and np.array_equal(la, lb)
    assert np.array_equal(a.read_params(), b.read_params())
    assert np.array_equal(a.read_params(which=1), b.read_params(which=1))
    for j in (0, 1):
        assert np.array_equal(a.read_state(0, a.n_units, j), b.read_state(0, b.n_units, j))

