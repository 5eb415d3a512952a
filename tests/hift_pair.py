"""Helpers of the GPU parity tests: build the oracle and the GPU model from the same seeded
inputs and run both over the same batches."""
import numpy as np

from hift_inputs import init_params, make_batch, model_config
from oracle import hift_oracle as O


def spec_of(cfg):
    return [(n, s, k) for n, s, k, _u in O.param_tensors(cfg)]


_LAST_WEIGHTS = {}


def initial_weights(cfg, seed, jitter=0.0):
    """init_params of a configuration, the most recent result kept: several tests build the same large model (the 7B
    widths at depth 2 are 667 M values, seconds to draw) and only read the vector."""
    import json
    layout = {k: v for k, v in cfg.items() if k not in ("unfused", "norm_eps", "rope_base")}
    key = (json.dumps(layout, sort_keys=True, default=str), seed, jitter)
    if _LAST_WEIGHTS.get("key") != key:
        _LAST_WEIGHTS.clear()
        theta0 = init_params(seed, spec_of(cfg), bf16_exact=(cfg["dtype"] == 1), jitter=jitter)
        theta0.setflags(write=False)
        _LAST_WEIGHTS.update(key=key, val=theta0)
    return _LAST_WEIGHTS["val"]


def make_pair(wl, seed=0, m=None, strategy=None, opt=None, state_on_host=0, batch=None, seq=None,
              jitter=0.0, sched_seed=17, master_on_host=0, no_packed_copies=0, unfused=0, **cfg_over):
    """Returns (oracle, gpu_model, theta0).  Weights are bf16-exact when the GPU model is bf16."""
    import paper_2401_15207_amd as H
    cfg = model_config(wl, **cfg_over)
    opt = dict(opt or wl["opt"])
    m = m or wl["m"]
    strategy = strategy or wl["strategy"]
    b, s = batch or wl["batch"], seq or wl["seq"]
    theta0 = initial_weights(cfg, seed, jitter)
    orc = O.HiftOracle(cfg, opt, theta0.astype(np.float64), half_weights=(cfg["dtype"] == 1))
    gpu = H.HiftModel(cfg, opt, m, b, s, init_params=theta0, state_on_host=state_on_host,
                      master_on_host=master_on_host, no_packed_copies=no_packed_copies, unfused=unfused)
    ko = orc.set_group_schedule(strategy, m, sched_seed)
    kg = gpu.set_group_schedule(strategy, m, sched_seed)
    assert ko == kg
    return orc, gpu, theta0


def to_dev(tok, lab):
    import torch
    return (torch.from_numpy(np.ascontiguousarray(tok)).cuda(), torch.from_numpy(np.ascontiguousarray(lab)).cuda())


def record(test, **fields):
    """Measured parity figures: printed (pytest -s shows them) and appended, one JSON object per line, to
    gpurun_out/parity_measured.jsonl when that scratch folder can be written."""
    import json
    import os
    rec = dict(test=test, **{k: (float(v) if isinstance(v, (np.floating, float)) else v) for k, v in fields.items()})
    line = json.dumps(rec)
    print("PARITY", line, flush=True)
    try:
        d = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out")
        os.makedirs(d, exist_ok=True)
        with open(os.path.join(d, "parity_measured.jsonl"), "a") as f:
            f.write(line + "\n")
    except OSError:
        pass


def rel_l2(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    den = np.linalg.norm(b)
    return np.linalg.norm(a - b) / den if den > 0 else np.linalg.norm(a)


def run_steps(orc, gpu, wl, seed, steps, batch=None, seq=None):
    """Runs `steps` scheduled steps on both sides; yields per step
    (t, gid, loss_oracle, loss_gpu, UpdateCheck, theta_before_gpu)."""
    for t in range(1, steps + 1):
        gid = orc.schedule_group_at(t)
        assert gid == gpu.schedule_group_at(t)
        tok, lab = make_batch(wl, seed, t, batch, seq)
        dtok, dlab = to_dev(tok, lab)
        tb_g = gpu.read_params()
        chk = UpdateCheck(orc, gid)
        lo = orc.step(tok, lab, gid)
        lg = gpu.step(dtok, dlab, gid)
        yield t, gid, lo, lg, chk, tb_g


def oracle_update(opt, theta, g, s1, s2, tg, dm):
    """New parameters of a slice under the oracle's optimizer formulas; inputs are not modified."""
    th, a, b = theta.copy(), s1.copy(), s2.copy()
    if opt["kind"] == "adamw":
        O.adamw_update(th, g, a, b, tg, opt["lr"], opt["beta1"], opt["beta2"], opt["eps"], opt["weight_decay"], dm)
    elif opt["kind"] == "adagrad":
        a = np.maximum(a, 0.0)     # a perturbed accumulator stays a sum of squares
        O.adagrad_update(th, g, a, opt["lr"], opt["eps"], opt["weight_decay"], dm)
    else:
        O.sgd_update(th, g, a, tg, opt["lr"], opt["momentum"], opt["weight_decay"], dm)
    return th


class UpdateCheck:
    """Tolerance of an optimizer update that follows from a tolerance on the gradient.

    The gradient of the GPU path may differ from the oracle's by tol * (|g_i| + rms of the
    gradient of the tensor that holds element i) per element.  An adaptive optimizer divides by a function of g, so the same relative tolerance
    does not carry over to the update where |g_i| is tiny (AdamW's first step is
    lr * g / (|g| + eps)).  The allowed error of element i is therefore the change of the
    oracle's own update when g_i moves by that amount, plus tol * |update_i|, plus the
    resolution of fp32 storage of theta.  In bf16 mode a small fraction of elements
    (max_outlier_frac) may exceed it: sums of many terms of both signs lose more than the
    typical relative error in the few elements where they nearly cancel."""

    def __init__(self, orc, gid):
        self.orc, self.gid = orc, gid
        self.lo, self.hi = orc.group_range(gid)
        sl = slice(self.lo, self.hi)
        self.th0 = orc.theta[sl].copy()
        self.s1, self.s2 = orc.state1[sl].copy(), orc.state2[sl].copy()
        self.tg = orc.group_steps[gid] + 1

    def check(self, theta_gpu_before, theta_gpu_after, tol, store_eps=1.2e-7, max_outlier_frac=0.0, max_elements=1 << 23):
        """theta_gpu_before / theta_gpu_after: the whole parameter vector, or (group_only=True implied by their size)
        the group's slice alone.  Groups of more than max_elements parameters are checked element by element on an
        evenly strided subset of that size (the bound is evaluated by running the oracle's optimizer several times,
        which for a group of 600 M parameters would take longer than the step it checks); the relative L2 figures
        are taken over the whole group."""
        orc = self.orc
        sl = slice(self.lo, self.hi)
        n = self.hi - self.lo
        if theta_gpu_before.size == n:
            before_g, after_g = theta_gpu_before, theta_gpu_after
        else:
            before_g, after_g = theta_gpu_before[sl], theta_gpu_after[sl]
        g = orc.last_grad[sl]
        dm = orc.decay_mask[sl]
        def tensor_rms(v):      # rms of v over the tensor each element belongs to
            out, off = np.zeros_like(v), 0
            for _n, shape, _k, _u in O.param_tensors(orc.cfg):
                cnt = int(np.prod(shape))
                a, b = max(off, self.lo), min(off + cnt, self.hi)
                if a < b:
                    seg = v[a - self.lo:b - self.lo]
                    out[a - self.lo:b - self.lo] = np.sqrt(np.mean(seg * seg))
                off += cnt
            return out

        up0_all = orc.theta[sl] - self.th0
        upg_all = after_g.astype(np.float64) - before_g.astype(np.float64)
        den = np.linalg.norm(up0_all)
        self.update_rel_l2 = float(np.linalg.norm(upg_all - up0_all) / den) if den > 0 else float(np.linalg.norm(upg_all))
        ref_after = orc.theta[sl]
        self.weights_rel_l2 = float(np.linalg.norm(after_g.astype(np.float64) - ref_after) / np.linalg.norm(ref_after))
        # the stored first-order state (moment / momentum buffer) carries the same relative
        # uncertainty as the gradients it was built from
        ix = slice(None, None, max(1, -(-n // max_elements)))
        delta = (tol * (np.abs(g) + tensor_rms(g)))[ix]
        delta_s = (tol * (np.abs(self.s1) + tensor_rms(self.s1)))[ix]
        th0, g, s1, s2, dm = self.th0[ix], g[ix], self.s1[ix], self.s2[ix], dm[ix]
        up0, upg = up0_all[ix], upg_all[ix]
        slack = np.zeros_like(g)
        for sg in (+1, -1):
            for ss in ((+1, -1) if self.tg > 1 else (0,)):
                up = oracle_update(orc.opt, th0, g + sg * delta, s1 + ss * delta_s, s2, self.tg, dm) - th0
                slack = np.maximum(slack, np.abs(up - up0))
        rel = tol if self.tg == 1 else 2 * tol     # later updates also divide by an uncertain second moment
        bound = 1.5 * slack + rel * np.abs(up0) + store_eps * np.abs(th0)
        err = np.abs(upg - up0)
        worst = int(np.argmax(err - bound))
        frac = float(np.mean(err > bound))
        self.outlier_frac = frac
        return frac <= max_outlier_frac, (frac, worst, float(err[worst]), float(bound[worst]), float(g[worst]))
