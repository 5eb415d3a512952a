"""CPU oracle of one HiFT training step (hierarchical fine-tuning, arxiv 2401.15207).

TEST INFRASTRUCTURE ONLY.  Nothing of the GPU library imports this file and this file imports
nothing of it.  It is called by the test-suite, by the smoke check and by the benchmark's
`cpu_baseline` leg.

What it computes.  A HiFT step with active group i minimises the loss over the masked
parameters beta_i o theta and leaves (1 - beta_i) o theta untouched (section 3, Eq. 2-3).
Freezing removes work but not results, so the oracle is the plain definition written out:

  1. full forward pass of the whole model,
  2. full reverse-mode gradient of the mean loss with respect to ALL parameters,
  3. keep only the slice of the active group (the mask beta_i),
  4. apply the optimizer to that slice with that group's own state and step counter,
  5. leave every other value untouched.

There is no truncation, no offload and no prefetch here.  All arithmetic is numpy in float64
(a float32 instance is possible through `dtype`).  numpy `matmul` serves as the matrix-product
step and scipy's `erf` as the error function.

Mixed precision (appendix "Mixing Precision": a half-precision model with a single-precision
backup of the weights, of which only the active group's part is touched per step).  With
`half_weights=True` the loss and its gradient are evaluated at the bf16 rounding
(round-to-nearest-even) of the master weights, and the update is applied to the master
weights; all arithmetic stays float64.  This models the one place where the precision of the
method, not of the arithmetic, changes the result: an update smaller than half a bf16 spacing
leaves the forward weights unchanged until enough updates accumulate.

Layer units, groups and visiting order (section 3 "Notation", Algorithm 1, appendix
"Implementation Details"): unit 0 = all embeddings including the position table, units 1..L =
hidden layers, unit L+1 = all head parameters; n = L + 2.  Groups are m consecutive units,
k = n/m if m divides n else floor(n/m) + 1; the short group is the top one.  bottom2up visits
groups 0..k-1, top2down k-1..0, random a permutation drawn once before training and then kept.
Step t (1-based) uses order[(t-1) mod k].  The learning rate may change only when all groups
have been visited once (Algorithm 1, learning-rate branch): `cycles_done` reports floor(t/k).

Readings of points the paper leaves open are listed in the repository's design notes; the ones
that matter here: final norm belongs to the head unit, embedding LayerNorm to the embedding
unit; AdamW bias correction uses a per-group update counter; weight decay applies to tensors
with two or more dimensions; eps 1e-8 (AdamW), 1e-10 (AdaGrad, zero initial accumulator);
SGD momentum without dampening or Nesterov, first buffer = first gradient; erf-GELU; RoPE pairs
(i, i + hd/2) with base 10000; no dropout, clipping or accumulation; embeddings untied unless
the configuration sets `tie_embeddings` (GPT-2 / OPT of section 4.1 share the token table with the
output matrix): the shared matrix then belongs to the embeddings unit, the head unit keeps the
final norm alone, and the table's gradient is the sum over its two uses.

Pins (tests/test_oracle_*.py): central finite differences of every tensor in float64,
PyTorch-autograd gradients of an independently written forward, frozen-parameter bit
identity, single-group == full step, hand-computed optimizer updates, integer tables of the
grouping, printed parameter counts (34 units at 7B; peak trainable share 2.44 % at 13B),
textbook special cases of softmax / cross-entropy / RoPE / normalisation / attention.
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf as _erf

ARCH_PRELN_DECODER = 0    # learned positions, LayerNorm (pre), GELU, biases, causal LM
ARCH_POSTLN_ENCODER = 1   # learned positions, LayerNorm (post), GELU, biases, classifier on token 0
ARCH_RMS_ROPE_DECODER = 2  # RMSNorm (pre), RoPE, SwiGLU, no biases, causal LM

KIND_MATRIX, KIND_GAIN, KIND_BIAS = 0, 1, 2
STRATEGIES = ("bottom2up", "top2down", "random")


# ----------------------------------------------------------------------------------------
# parameter layout: units and tensors (appendix "Implementation Details": layering principle)
# ----------------------------------------------------------------------------------------
def param_tensors(cfg: dict):
    """Canonical tensor list [(name, shape, kind, unit)], in storage order."""
    a, L, d, f, V = cfg["arch"], cfg["n_layers"], cfg["d_model"], cfg["d_ffn"], cfg["vocab"]
    tied = bool(cfg.get("tie_embeddings", 0))   # decoders only: the output matrix is the token table (unit 0)
    if tied and a == ARCH_POSTLN_ENCODER:
        raise ValueError("tie_embeddings applies to the decoders")
    out = []
    if a == ARCH_PRELN_DECODER:
        out += [("tok_emb", (V, d), KIND_MATRIX, 0), ("pos_emb", (cfg["max_seq"], d), KIND_MATRIX, 0)]
        for l in range(L):
            u, p = l + 1, f"l{l}."
            out += [(p + "ln1_g", (d,), KIND_GAIN, u), (p + "ln1_b", (d,), KIND_BIAS, u),
                    (p + "wqkv", (3 * d, d), KIND_MATRIX, u), (p + "bqkv", (3 * d,), KIND_BIAS, u),
                    (p + "wo", (d, d), KIND_MATRIX, u), (p + "bo", (d,), KIND_BIAS, u),
                    (p + "ln2_g", (d,), KIND_GAIN, u), (p + "ln2_b", (d,), KIND_BIAS, u),
                    (p + "w1", (f, d), KIND_MATRIX, u), (p + "b1", (f,), KIND_BIAS, u),
                    (p + "w2", (d, f), KIND_MATRIX, u), (p + "b2", (d,), KIND_BIAS, u)]
        out += [("lnf_g", (d,), KIND_GAIN, L + 1), ("lnf_b", (d,), KIND_BIAS, L + 1)]
        if not tied:
            out += [("whead", (V, d), KIND_MATRIX, L + 1)]
    elif a == ARCH_POSTLN_ENCODER:
        out += [("tok_emb", (V, d), KIND_MATRIX, 0), ("pos_emb", (cfg["max_seq"], d), KIND_MATRIX, 0),
                ("lne_g", (d,), KIND_GAIN, 0), ("lne_b", (d,), KIND_BIAS, 0)]
        for l in range(L):
            u, p = l + 1, f"l{l}."
            out += [(p + "wqkv", (3 * d, d), KIND_MATRIX, u), (p + "bqkv", (3 * d,), KIND_BIAS, u),
                    (p + "wo", (d, d), KIND_MATRIX, u), (p + "bo", (d,), KIND_BIAS, u),
                    (p + "ln1_g", (d,), KIND_GAIN, u), (p + "ln1_b", (d,), KIND_BIAS, u),
                    (p + "w1", (f, d), KIND_MATRIX, u), (p + "b1", (f,), KIND_BIAS, u),
                    (p + "w2", (d, f), KIND_MATRIX, u), (p + "b2", (d,), KIND_BIAS, u),
                    (p + "ln2_g", (d,), KIND_GAIN, u), (p + "ln2_b", (d,), KIND_BIAS, u)]
        C = cfg["n_classes"]
        out += [("wc", (C, d), KIND_MATRIX, L + 1), ("bc", (C,), KIND_BIAS, L + 1)]
    elif a == ARCH_RMS_ROPE_DECODER:
        out += [("tok_emb", (V, d), KIND_MATRIX, 0)]
        for l in range(L):
            u, p = l + 1, f"l{l}."
            out += [(p + "g1", (d,), KIND_GAIN, u), (p + "wqkv", (3 * d, d), KIND_MATRIX, u),
                    (p + "wo", (d, d), KIND_MATRIX, u), (p + "g2", (d,), KIND_GAIN, u),
                    (p + "wgu", (2 * f, d), KIND_MATRIX, u), (p + "wd", (d, f), KIND_MATRIX, u)]
        out += [("gf", (d,), KIND_GAIN, L + 1)]
        if not tied:
            out += [("whead", (V, d), KIND_MATRIX, L + 1)]
    else:
        raise ValueError("unknown arch")
    return out


def n_units(cfg: dict) -> int:
    return cfg["n_layers"] + 2


def unit_ranges(cfg: dict):
    """[(offset, count)] of every unit in the flat parameter vector."""
    n = n_units(cfg)
    cnt = [0] * n
    for _name, shape, _kind, u in param_tensors(cfg):
        cnt[u] += int(np.prod(shape))
    off, out = 0, []
    for c in cnt:
        out.append((off, c))
        off += c
    return out


def n_params(cfg: dict) -> int:
    return sum(c for _o, c in unit_ranges(cfg))


# ----------------------------------------------------------------------------------------
# memory accounting (appendix "Memory Analysis")
# ----------------------------------------------------------------------------------------
STATE_ARRAYS = {"adamw": 2, "adagrad": 1, "sgd": 0, "sgdm": 1}


def memory_model(cfg: dict, m: int, state_arrays: int = 2, bytes_per: int = 4) -> dict:
    """Bytes held by weights, gradients and optimizer state (the three terms of the appendix).
    zeta1 = weights, zeta2 = state_arrays * zeta1, zeta3 = zeta1 (gradients of what is updated).
    Full fine-tuning keeps all three whole; HiFT keeps the weights whole and, of the other two, only
    the active group's share: averaged over k equal groups that is zeta1 + (zeta2 + zeta3) / k, which
    for AdamW is (k + 3) / k * zeta1; the peak over the cycle uses the largest group instead."""
    ur = unit_ranges(cfg)
    n = len(ur)
    k = n_groups(n, m)
    P = sum(c for _o, c in ur)
    peak = max(sum(ur[u][1] for u in group_units(n, m, j)) for j in range(k))
    z1 = bytes_per * P
    z2, z3 = state_arrays * z1, z1
    return {
        "k": k, "n_params": P, "peak_trainable": peak,
        "zeta1": z1, "zeta_fpft": z1 + z2 + z3,
        "zeta_hift": z1 + (z2 + z3) / k,
        "zeta_hift_peak": z1 + (state_arrays + 1) * bytes_per * peak,
        "delta": (z1 + z2 + z3) - (z1 + (z2 + z3) / k),
    }


# ----------------------------------------------------------------------------------------
# grouping and visiting order (section 3 "Notation"; Algorithm 1 initialisation, steps c-d)
# ----------------------------------------------------------------------------------------
def n_groups(n: int, m: int) -> int:
    if m < 1:
        raise ValueError("m must be >= 1")
    return n // m if n % m == 0 else n // m + 1


def group_units(n: int, m: int, j: int):
    """Units of group j: m consecutive units, the top group may be short."""
    return list(range(j * m, min((j + 1) * m, n)))


def lr_at_cycle(kind: str, base_lr: float, warmup_cycles: int, total_cycles: int, cycle: int) -> float:
    """Learning rate in force during cycle `cycle` (0-based count of completed sweeps over all groups).
    The delayed update strategy (section 3, "delayed learning rate update") advances the scheduler once per
    sweep instead of once per step, so the usual schedules are evaluated at the cycle index:
      constant: base_lr
      linear:   base_lr * cycle / warmup_cycles                       while cycle < warmup_cycles
                base_lr * max(0, (total - cycle) / (total - warmup))  afterwards (the warm-up/linear-decay
                schedule of the paper's hyper-parameter tables)."""
    if kind == "constant":
        return base_lr
    if kind != "linear":
        raise ValueError("unknown schedule")
    if cycle < warmup_cycles:
        return base_lr * cycle / max(1, warmup_cycles)
    return base_lr * max(0.0, (total_cycles - cycle) / max(1, total_cycles - warmup_cycles))


def splitmix64(state: int):
    """One draw of the SplitMix64 generator (Steele, Lea, Flood 2014): returns (value, new state)."""
    mask = (1 << 64) - 1
    state = (state + 0x9E3779B97F4A7C15) & mask
    z = state
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
    return z ^ (z >> 31), state


def group_order(k: int, strategy: str, seed: int = 0):
    """Visiting order of the k groups.  random: Fisher-Yates from the top index down, the
    swap partner of index i is (SplitMix64 draw) mod (i + 1); drawn once and then kept."""
    if strategy == "bottom2up":
        return list(range(k))
    if strategy == "top2down":
        return list(range(k - 1, -1, -1))
    if strategy == "random":
        order, s = list(range(k)), int(seed) & ((1 << 64) - 1)
        for i in range(k - 1, 0, -1):
            r, s = splitmix64(s)
            j = r % (i + 1)
            order[i], order[j] = order[j], order[i]
        return order
    raise ValueError("unknown strategy")


# ----------------------------------------------------------------------------------------
# building blocks: forward and adjoint of each operation (textbook definitions)
# ----------------------------------------------------------------------------------------
def layernorm_fwd(x, g, b, eps):
    mu = x.mean(-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xh = xc * rstd
    return xh * g + b, (xh, rstd)


def layernorm_bwd(dy, cache, g):
    xh, rstd = cache
    dg = (dy * xh).reshape(-1, xh.shape[-1]).sum(0)
    db = dy.reshape(-1, xh.shape[-1]).sum(0)
    dxh = dy * g
    dx = rstd * (dxh - dxh.mean(-1, keepdims=True) - xh * (dxh * xh).mean(-1, keepdims=True))
    return dx, dg, db


def rmsnorm_fwd(x, g, eps):
    ms = (x * x).mean(-1, keepdims=True)
    rstd = 1.0 / np.sqrt(ms + eps)
    xh = x * rstd
    return xh * g, (xh, rstd)


def rmsnorm_bwd(dy, cache, g):
    xh, rstd = cache
    dg = (dy * xh).reshape(-1, xh.shape[-1]).sum(0)
    dxh = dy * g
    dx = rstd * (dxh - xh * (dxh * xh).mean(-1, keepdims=True))
    return dx, dg


def gelu_cdf(x):
    """Phi(x), the standard normal distribution function."""
    return 0.5 * (1.0 + _erf(x / math.sqrt(2.0)))


def gelu_fwd(x, cdf=None):
    """x Phi(x).  cdf: Phi(x) if the caller has it already (the error function is the slow part)."""
    return x * (gelu_cdf(x) if cdf is None else cdf)


def gelu_bwd(dy, x, cdf=None):
    """dy (Phi(x) + x phi(x))."""
    cdf = gelu_cdf(x) if cdf is None else cdf
    pdf = np.exp(-0.5 * x * x) / math.sqrt(2.0 * math.pi)
    return dy * (cdf + x * pdf)


def silu(x):
    return x / (1.0 + np.exp(-x))


def swiglu_fwd(g, u):
    return silu(g) * u


def swiglu_bwd(da, g, u):
    s = 1.0 / (1.0 + np.exp(-g))
    dsilu = s * (1.0 + g * (1.0 - s))
    return da * u * dsilu, da * g * s


def rope_angles(S, hd, base, dtype):
    """cos, sin of shape [S, hd/2]: angle(p, i) = p * base^(-2i/hd)."""
    i = np.arange(hd // 2, dtype=np.float64)
    inv = base ** (-2.0 * i / hd)
    ang = np.arange(S, dtype=np.float64)[:, None] * inv[None, :]
    return np.cos(ang).astype(dtype), np.sin(ang).astype(dtype)


def rope_fwd(x, cos, sin):
    """x [B, H, S, hd]; rotates the pair (i, i + hd/2) by angle(p, i)."""
    h = x.shape[-1] // 2
    x1, x2 = x[..., :h], x[..., h:]
    return np.concatenate([x1 * cos - x2 * sin, x1 * sin + x2 * cos], -1)


def rope_bwd(dy, cos, sin):
    """Adjoint of a rotation = rotation by the negative angle."""
    h = dy.shape[-1] // 2
    d1, d2 = dy[..., :h], dy[..., h:]
    return np.concatenate([d1 * cos + d2 * sin, -d1 * sin + d2 * cos], -1)


def softmax_lastdim(s):
    s = s - s.max(-1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(-1, keepdims=True)


def attention_fwd(q, k, v, causal):
    """q, k, v [B, H, S, hd] -> softmax(q k^T / sqrt(hd) + mask) v."""
    hd, S = q.shape[-1], q.shape[-2]
    s = np.matmul(q, np.swapaxes(k, -1, -2)) / math.sqrt(hd)
    if causal:
        s = np.where(np.tril(np.ones((S, S), dtype=bool)), s, -np.inf)
    p = softmax_lastdim(s)
    return np.matmul(p, v), p


def attention_bwd(dctx, q, k, v, p):
    hd = q.shape[-1]
    dv = np.matmul(np.swapaxes(p, -1, -2), dctx)
    dp = np.matmul(dctx, np.swapaxes(v, -1, -2))
    ds = p * (dp - (dp * p).sum(-1, keepdims=True))
    dq = np.matmul(ds, k) / math.sqrt(hd)
    dk = np.matmul(np.swapaxes(ds, -1, -2), q) / math.sqrt(hd)
    return dq, dk, dv


def cross_entropy_fwd(logits, labels):
    """Mean over rows with label >= 0 of -log softmax(logits)[label].
    Returns loss and d loss / d logits.  A batch without a single target (sequences of one token: the paper does
    not treat it) has loss 0 and gradient 0: the mean over no rows is taken as the empty sum."""
    z = logits - logits.max(-1, keepdims=True)
    lse = np.log(np.exp(z).sum(-1, keepdims=True))
    logp = z - lse
    valid = labels >= 0
    nv = int(valid.sum())
    if nv == 0:
        return 0.0, np.zeros_like(logp)
    rows = np.nonzero(valid)[0]
    loss = -logp[rows, labels[rows]].sum() / nv
    dlogits = np.exp(logp)
    dlogits[rows, labels[rows]] -= 1.0
    dlogits[~valid] = 0.0
    dlogits /= nv
    return loss, dlogits


# ----------------------------------------------------------------------------------------
# model: forward + full backward
# ----------------------------------------------------------------------------------------
class _Params:
    """Views of the flat vector by tensor name."""

    def __init__(self, cfg, flat):
        self.views, off = {}, 0
        for name, shape, _kind, _u in param_tensors(cfg):
            n = int(np.prod(shape))
            self.views[name] = flat[off:off + n].reshape(shape)
            off += n
        assert off == flat.size

    def __getitem__(self, k):
        return self.views[k]


def _split_heads(x, B, S, H):
    return x.reshape(B, S, H, -1).transpose(0, 2, 1, 3)


def _merge_heads(x):
    B, H, S, hd = x.shape
    return x.transpose(0, 2, 1, 3).reshape(B * S, H * hd)


def loss_and_grad(cfg: dict, flat: np.ndarray, tokens: np.ndarray, labels: np.ndarray,
                  need_grad: bool = True):
    """Mean loss of the batch and, if asked, its gradient with respect to every parameter
    (flat, canonical order).  tokens int [B, S]; labels int [B, S] (decoders, -1 = no target)
    or int [B] (encoder)."""
    a, L, d, H = cfg["arch"], cfg["n_layers"], cfg["d_model"], cfg["n_heads"]
    eps = cfg["norm_eps"]
    dt = flat.dtype
    P = _Params(cfg, flat)
    B, S = tokens.shape
    T = B * S
    hd = d // H
    tok = tokens.reshape(-1).astype(np.int64)
    pos = np.tile(np.arange(S), B)
    causal = a != ARCH_POSTLN_ENCODER
    pre_ln = a != ARCH_POSTLN_ENCODER
    rms = a == ARCH_RMS_ROPE_DECODER
    if rms:
        cos, sin = rope_angles(S, hd, cfg["rope_base"], dt)

    def norm_fwd(x, name_g, name_b):
        return rmsnorm_fwd(x, P[name_g], eps) if rms else layernorm_fwd(x, P[name_g], P[name_b], eps)

    # ---- forward ----
    cache = []
    if a == ARCH_RMS_ROPE_DECODER:
        x = P["tok_emb"][tok].copy()
    else:
        x = P["tok_emb"][tok] + P["pos_emb"][pos]
        if a == ARCH_POSTLN_ENCODER:
            x, emb_ln = layernorm_fwd(x, P["lne_g"], P["lne_b"], eps)

    for l in range(L):
        p = f"l{l}."
        c = {}
        # attention sub-layer
        if pre_ln:
            h1, c["n1"] = norm_fwd(x, p + ("g1" if rms else "ln1_g"), p + "ln1_b")
        else:
            h1 = x
        c["h1"] = h1
        qkv = h1 @ P[p + "wqkv"].T
        if not rms:
            qkv = qkv + P[p + "bqkv"]
        q, k, v = (_split_heads(qkv[:, i * d:(i + 1) * d], B, S, H) for i in range(3))
        if rms:
            q, k = rope_fwd(q, cos, sin), rope_fwd(k, cos, sin)
        ctx4, prob = attention_fwd(q, k, v, causal)
        c["q"], c["k"], c["v"], c["p"] = q, k, v, prob
        ctx = _merge_heads(ctx4)
        c["ctx"] = ctx
        ao = ctx @ P[p + "wo"].T
        if not rms:
            ao = ao + P[p + "bo"]
        x = x + ao
        if not pre_ln:
            x, c["n1"] = layernorm_fwd(x, P[p + "ln1_g"], P[p + "ln1_b"], eps)
        # feed-forward sub-layer
        if pre_ln:
            h2, c["n2"] = norm_fwd(x, p + ("g2" if rms else "ln2_g"), p + "ln2_b")
        else:
            h2 = x
        c["h2"] = h2
        if rms:
            gu = h2 @ P[p + "wgu"].T
            f = gu.shape[1] // 2
            c["g"], c["u"] = gu[:, :f], gu[:, f:]
            act = swiglu_fwd(c["g"], c["u"])
            fo = act @ P[p + "wd"].T
        else:
            pre = h2 @ P[p + "w1"].T + P[p + "b1"]
            c["pre"] = pre
            c["cdf"] = gelu_cdf(pre)          # kept for the backward pass: the same values, evaluated once
            act = gelu_fwd(pre, c["cdf"])
            fo = act @ P[p + "w2"].T + P[p + "b2"]
        c["act"] = act
        x = x + fo
        if not pre_ln:
            x, c["n2"] = layernorm_fwd(x, P[p + "ln2_g"], P[p + "ln2_b"], eps)
        cache.append(c)

    if a == ARCH_POSTLN_ENCODER:
        xc = x.reshape(B, S, d)[:, 0, :]
        logits = xc @ P["wc"].T + P["bc"]
        loss, dlogits = cross_entropy_fwd(logits, labels.reshape(-1).astype(np.int64))
    else:
        xf, nf = norm_fwd(x, "gf" if rms else "lnf_g", "lnf_b")
        head = "tok_emb" if cfg.get("tie_embeddings", 0) else "whead"
        logits = xf @ P[head].T
        loss, dlogits = cross_entropy_fwd(logits, labels.reshape(-1).astype(np.int64))
    if not need_grad:
        return float(loss), None

    # ---- backward (all parameters) ----
    gflat = np.zeros_like(flat)
    G = _Params(cfg, gflat)
    if a == ARCH_POSTLN_ENCODER:
        G["wc"][...] = dlogits.T @ xc
        G["bc"][...] = dlogits.sum(0)
        dxc = dlogits @ P["wc"]
        dx = np.zeros((B, S, d), dtype=dt)
        dx[:, 0, :] = dxc
        dx = dx.reshape(T, d)
    else:
        G[head][...] = dlogits.T @ xf      # tied: the token table's gradient starts with its use as output matrix
        dxf = dlogits @ P[head]
        if rms:
            dx, G["gf"][...] = rmsnorm_bwd(dxf, nf, P["gf"])
        else:
            dx, G["lnf_g"][...], G["lnf_b"][...] = layernorm_bwd(dxf, nf, P["lnf_g"])

    for l in range(L - 1, -1, -1):
        p = f"l{l}."
        c = cache[l]
        # feed-forward sub-layer
        if not pre_ln:
            dx, G[p + "ln2_g"][...], G[p + "ln2_b"][...] = layernorm_bwd(dx, c["n2"], P[p + "ln2_g"])
        dfo = dx
        if rms:
            G[p + "wd"][...] = dfo.T @ c["act"]
            dact = dfo @ P[p + "wd"]
            dg, du = swiglu_bwd(dact, c["g"], c["u"])
            dgu = np.concatenate([dg, du], 1)
            G[p + "wgu"][...] = dgu.T @ c["h2"]
            dh2 = dgu @ P[p + "wgu"]
        else:
            G[p + "w2"][...] = dfo.T @ c["act"]
            G[p + "b2"][...] = dfo.sum(0)
            dact = dfo @ P[p + "w2"]
            dpre = gelu_bwd(dact, c["pre"], c["cdf"])
            G[p + "w1"][...] = dpre.T @ c["h2"]
            G[p + "b1"][...] = dpre.sum(0)
            dh2 = dpre @ P[p + "w1"]
        if pre_ln:
            if rms:
                dn, G[p + "g2"][...] = rmsnorm_bwd(dh2, c["n2"], P[p + "g2"])
            else:
                dn, G[p + "ln2_g"][...], G[p + "ln2_b"][...] = layernorm_bwd(dh2, c["n2"], P[p + "ln2_g"])
            dx = dx + dn
        else:
            dx = dx + dh2
        # attention sub-layer
        if not pre_ln:
            dx, G[p + "ln1_g"][...], G[p + "ln1_b"][...] = layernorm_bwd(dx, c["n1"], P[p + "ln1_g"])
        dao = dx
        G[p + "wo"][...] = dao.T @ c["ctx"]
        if not rms:
            G[p + "bo"][...] = dao.sum(0)
        dctx = _split_heads(dao @ P[p + "wo"], B, S, H)
        dq, dk, dv = attention_bwd(dctx, c["q"], c["k"], c["v"], c["p"])
        if rms:
            dq, dk = rope_bwd(dq, cos, sin), rope_bwd(dk, cos, sin)
        dqkv = np.concatenate([_merge_heads(dq), _merge_heads(dk), _merge_heads(dv)], 1)
        G[p + "wqkv"][...] = dqkv.T @ c["h1"]
        if not rms:
            G[p + "bqkv"][...] = dqkv.sum(0)
        dh1 = dqkv @ P[p + "wqkv"]
        if pre_ln:
            if rms:
                dn, G[p + "g1"][...] = rmsnorm_bwd(dh1, c["n1"], P[p + "g1"])
            else:
                dn, G[p + "ln1_g"][...], G[p + "ln1_b"][...] = layernorm_bwd(dh1, c["n1"], P[p + "ln1_g"])
            dx = dx + dn
        else:
            dx = dx + dh1

    # embeddings
    if a == ARCH_POSTLN_ENCODER:
        dx, G["lne_g"][...], G["lne_b"][...] = layernorm_bwd(dx, emb_ln, P["lne_g"])
    np.add.at(G["tok_emb"], tok, dx)
    if a != ARCH_RMS_ROPE_DECODER:
        np.add.at(G["pos_emb"], pos, dx)
    return float(loss), gflat


# ----------------------------------------------------------------------------------------
# optimizers on a slice (Algorithm 1 step g and the update inside the backward step)
# ----------------------------------------------------------------------------------------
def adamw_update(theta, g, m, v, t, lr, beta1, beta2, eps, wd, decay_mask):
    """Decoupled weight decay, then the bias-corrected Adam step; t = 1 on the first update."""
    theta *= (1.0 - lr * wd * decay_mask)
    m[...] = beta1 * m + (1.0 - beta1) * g
    v[...] = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    theta -= lr * mhat / (np.sqrt(vhat) + eps)


def adagrad_update(theta, g, acc, lr, eps, wd, decay_mask):
    """Accumulate squared gradients; weight decay, if any, enters as L2 term of the gradient."""
    g = g + wd * decay_mask * theta
    acc += g * g
    theta -= lr * g / (np.sqrt(acc) + eps)


def sgd_update(theta, g, buf, t, lr, momentum, wd, decay_mask):
    """SGD; with momentum mu > 0: b <- g on the first update, b <- mu b + g afterwards."""
    g = g + wd * decay_mask * theta
    if momentum > 0.0:
        if t == 1:
            buf[...] = g
        else:
            buf[...] = momentum * buf + g
        g = buf
    theta -= lr * g


def adafactor_update(theta, g, state, shape, t, lr, wd, decay, eps1=1e-30, clip=1.0, decay_rate=0.8):
    """Adafactor (Shazeer and Stern 2018, Algorithm 4 without momentum, with an external step
    size: no relative step, no parameter scaling).  One tensor per call; theta, g flat views.
      beta2_t = 1 - t^(-decay_rate)
      matrices [n, m]:  R <- beta2_t R + (1 - beta2_t) mean_j (G^2 + eps1)      (n values)
                        C <- beta2_t C + (1 - beta2_t) mean_i (G^2 + eps1)      (m values)
                        V_ij = R_i C_j / mean(R);   U = G / sqrt(V)
      vectors:          V <- beta2_t V + (1 - beta2_t) (G^2 + eps1);  U = G / sqrt(V)
      U <- U / max(1, rms(U) / clip);  theta <- theta - lr wd theta (decayed tensors) - lr U
    state: dict, created empty; holds "r", "c" (matrices) or "v" (vectors)."""
    b2 = 1.0 - float(t) ** (-decay_rate)
    if len(shape) >= 2:
        G = g.reshape(shape)
        sq = G * G + eps1
        if "r" not in state:
            state["r"], state["c"] = np.zeros(shape[0], theta.dtype), np.zeros(shape[1], theta.dtype)
        state["r"][...] = b2 * state["r"] + (1.0 - b2) * sq.mean(axis=1)
        state["c"][...] = b2 * state["c"] + (1.0 - b2) * sq.mean(axis=0)
        V = np.outer(state["r"], state["c"]) / state["r"].mean()
        U = (G / np.sqrt(V)).reshape(-1)
    else:
        if "v" not in state:
            state["v"] = np.zeros(g.shape, theta.dtype)
        state["v"][...] = b2 * state["v"] + (1.0 - b2) * (g * g + eps1)
        U = g / np.sqrt(state["v"])
    U = U / max(1.0, float(np.sqrt(np.mean(U * U))) / clip)
    if decay:
        theta -= lr * wd * theta
    theta -= lr * U


# ----------------------------------------------------------------------------------------
# low-rank adapters on the attention projections (the LoRA baseline of section 4.3, whose step
# time the paper sets beside HiFT's)
# ----------------------------------------------------------------------------------------
def lora_tensors(cfg: dict, rank: int):
    """Adapter tensors [(name, shape)], in storage order: per hidden layer A_q [r, d], A_v [r, d], B_q [d, r],
    B_v [d, r].  The query and value projections become W + (alpha / r) B A; everything else is frozen."""
    d = cfg["d_model"]
    out = []
    for l in range(cfg["n_layers"]):
        p = f"l{l}."
        out += [(p + "lora_aq", (rank, d)), (p + "lora_av", (rank, d)), (p + "lora_bq", (d, rank)), (p + "lora_bv", (d, rank))]
    return out


def lora_n_params(cfg: dict, rank: int) -> int:
    return sum(int(np.prod(shape)) for _n, shape in lora_tensors(cfg, rank))


def _lora_views(cfg, rank, flat):
    views, off = {}, 0
    for name, shape in lora_tensors(cfg, rank):
        n = int(np.prod(shape))
        views[name] = flat[off:off + n].reshape(shape)
        off += n
    return views


def lora_merge(cfg: dict, flat: np.ndarray, lora: np.ndarray, rank: int, alpha: float) -> np.ndarray:
    """The base parameters with every adapted projection replaced by W + (alpha / rank) B A (a copy)."""
    d, s = cfg["d_model"], alpha / rank
    merged = np.array(flat, copy=True)
    P, A = _Params(cfg, merged), _lora_views(cfg, rank, lora)
    for l in range(cfg["n_layers"]):
        p = f"l{l}."
        P[p + "wqkv"][0:d] += s * (A[p + "lora_bq"] @ A[p + "lora_aq"])
        P[p + "wqkv"][2 * d:3 * d] += s * (A[p + "lora_bv"] @ A[p + "lora_av"])
    return merged


def lora_loss_and_grad(cfg: dict, flat: np.ndarray, lora: np.ndarray, tokens, labels, rank: int, alpha: float):
    """Loss of the model with merged adapters and its gradient with respect to the adapters alone.  An adapter is a
    reparametrisation W' = W + s B A of a projection, so with G = d loss / d W' (from the full backward pass):
    d loss / d B = s G A^T and d loss / d A = s B^T G."""
    d, s = cfg["d_model"], alpha / rank
    loss, g = loss_and_grad(cfg, lora_merge(cfg, flat, lora, rank, alpha), tokens, labels)
    G, A = _Params(cfg, g), _lora_views(cfg, rank, lora)
    out = np.zeros_like(lora)
    D = _lora_views(cfg, rank, out)
    for l in range(cfg["n_layers"]):
        p = f"l{l}."
        for part, rows in (("q", slice(0, d)), ("v", slice(2 * d, 3 * d))):
            Gw = G[p + "wqkv"][rows]
            D[p + "lora_b" + part][...] = s * (Gw @ A[p + "lora_a" + part].T)
            D[p + "lora_a" + part][...] = s * (A[p + "lora_b" + part].T @ Gw)
    return loss, out


class LoraOracle:
    """A run that trains the adapters only (AdamW, no weight decay on anything but matrices -- every adapter is
    one); the base parameters never change.  With half_weights the loss is evaluated at the bf16 rounding of base and
    adapters, as the mixed-precision GPU path does."""

    def __init__(self, cfg, opt, params, lora, rank, alpha, half_weights=False):
        self.cfg, self.opt, self.rank, self.alpha, self.half = dict(cfg), dict(opt), rank, alpha, half_weights
        self.theta = np.array(params, dtype=np.float64).reshape(-1).copy()
        self.lora = np.array(lora, dtype=np.float64).reshape(-1).copy()
        assert self.theta.size == n_params(cfg) and self.lora.size == lora_n_params(cfg, rank)
        self.m, self.v = np.zeros_like(self.lora), np.zeros_like(self.lora)
        self.t = 0
        self.last_grad = None

    def step(self, tokens, labels) -> float:
        base = bf16_round(self.theta) if self.half else self.theta
        at = bf16_round(self.lora) if self.half else self.lora
        loss, g = lora_loss_and_grad(self.cfg, base, at, tokens, labels, self.rank, self.alpha)
        self.last_grad = g
        self.t += 1
        o = self.opt
        adamw_update(self.lora, g, self.m, self.v, self.t, o["lr"], o["beta1"], o["beta2"], o["eps"],
                     o["weight_decay"], np.ones_like(self.lora))
        return loss


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Nearest bfloat16 value (1 sign, 8 exponent, 7 fraction bits; ties to even), returned in
    x's dtype.  Values are first rounded to float32 (nearest even), whose upper 16 bits are the
    bfloat16 pattern."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    keep = (u >> 16) & 1
    u = ((u + 0x7FFF + keep) >> 16) << 16
    return u.astype(np.uint32).view(np.float32).astype(x.dtype).reshape(x.shape)


class HiftOracle:
    """State of a HiFT run: parameters, per-group optimizer state and counters."""

    def __init__(self, cfg: dict, opt: dict, params: np.ndarray, dtype=np.float64,
                 half_weights: bool = False):
        self.half_weights = half_weights
        self.cfg, self.opt = dict(cfg), dict(opt)
        self.theta = np.array(params, dtype=dtype).reshape(-1).copy()
        assert self.theta.size == n_params(cfg)
        self.n = n_units(cfg)
        self.units = unit_ranges(cfg)
        self.decay_mask = np.zeros_like(self.theta)
        off = 0
        for _name, shape, _kind, _u in param_tensors(cfg):
            c = int(np.prod(shape))
            if len(shape) >= 2:
                self.decay_mask[off:off + c] = 1.0
            off += c
        self.state1 = np.zeros_like(self.theta)   # AdamW m / AdaGrad accumulator / SGD buffer
        self.state2 = np.zeros_like(self.theta)   # AdamW v
        self.factored = {}                        # Adafactor: tensor name -> {"r","c"} or {"v"}
        self.k = None
        self.t = 0
        self.last_grad = None

    # -- Algorithm 1, initialisation --
    def set_group_schedule(self, strategy: str, m: int, seed: int = 0) -> int:
        self.m = m
        self.k = n_groups(self.n, m)
        self.order = group_order(self.k, strategy, seed)
        self.group_steps = [0] * self.k
        self.t = 0
        return self.k

    def schedule_group_at(self, t: int) -> int:
        return self.order[(t - 1) % self.k]

    @property
    def cycles_done(self) -> int:
        return self.t // self.k

    def set_lr(self, lr: float):
        self.opt["lr"] = lr

    def group_range(self, j: int):
        us = group_units(self.n, self.m, j)
        lo = self.units[us[0]][0]
        hi = self.units[us[-1]][0] + self.units[us[-1]][1]
        return lo, hi

    # -- Algorithm 1, steps e-k for one batch --
    def step(self, tokens, labels, group_id: int) -> float:
        if self.k is None or not (0 <= group_id < self.k):
            raise ValueError("bad group")
        if self.half_weights:
            # the half-precision model: kept between steps, since only the group updated last has changed
            if getattr(self, "_half", None) is None:
                self._half = bf16_round(self.theta)
            at = self._half
        else:
            at = self.theta
        loss, g = loss_and_grad(self.cfg, at, tokens, labels)
        self.last_grad = g
        lo, hi = self.group_range(group_id)
        self.group_steps[group_id] += 1
        tg = self.group_steps[group_id]
        o = self.opt
        th, gs, dm = self.theta[lo:hi], g[lo:hi], self.decay_mask[lo:hi]
        if o["kind"] == "adamw":
            adamw_update(th, gs, self.state1[lo:hi], self.state2[lo:hi], tg, o["lr"], o["beta1"],
                         o["beta2"], o["eps"], o["weight_decay"], dm)
        elif o["kind"] == "adagrad":
            adagrad_update(th, gs, self.state1[lo:hi], o["lr"], o["eps"], o["weight_decay"], dm)
        elif o["kind"] == "sgd":
            sgd_update(th, gs, self.state1[lo:hi], tg, o["lr"], o["momentum"], o["weight_decay"], dm)
        elif o["kind"] == "adafactor":
            off = 0
            for name, shape, _kind, _u in param_tensors(self.cfg):
                c = int(np.prod(shape))
                if lo <= off and off + c <= hi:
                    adafactor_update(self.theta[off:off + c], g[off:off + c], self.factored.setdefault(name, {}),
                                     shape, tg, o["lr"], o["weight_decay"], len(shape) >= 2)
                off += c
        else:
            raise ValueError("unknown optimizer")
        if self.half_weights:
            self._half[lo:hi] = bf16_round(self.theta[lo:hi])
        self.t += 1
        return loss

    def read_params(self, unit_lo: int = 0, unit_hi: int | None = None) -> np.ndarray:
        unit_hi = self.n if unit_hi is None else unit_hi
        lo = self.units[unit_lo][0]
        hi = self.units[unit_hi - 1][0] + self.units[unit_hi - 1][1]
        return self.theta[lo:hi].copy()
