"""Pins of the oracle's forward and backward: central finite differences in float64 and an
independent forward written with PyTorch CPU library routines, differentiated by autograd."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from hift_inputs import WORKLOADS, init_params, make_batch, model_config
from oracle import hift_oracle as O

SMALL = {
    0: dict(arch=0, n_layers=2, d_model=16, n_heads=2, d_ffn=40, vocab=29, max_seq=8, n_classes=0,
            norm_eps=1e-5, rope_base=10000.0, dtype=0),
    1: dict(arch=1, n_layers=2, d_model=16, n_heads=4, d_ffn=24, vocab=31, max_seq=10, n_classes=3,
            norm_eps=1e-5, rope_base=10000.0, dtype=0),
    2: dict(arch=2, n_layers=2, d_model=16, n_heads=2, d_ffn=24, vocab=37, max_seq=8, n_classes=0,
            norm_eps=1e-5, rope_base=10000.0, dtype=0),
}


def _setup(arch, seed=3, B=2, S=6, std=0.3, tied=0):
    cfg = dict(SMALL[arch], tie_embeddings=tied)
    spec = [(n, s, k) for n, s, k, _u in O.param_tensors(cfg)]
    theta = init_params(seed, spec, bf16_exact=False, std=std, jitter=0.2).astype(np.float64)
    wl = dict(cfg, batch=B, seq=S)
    tok, lab = make_batch(wl, seed, 0)
    return cfg, theta, tok, lab


@pytest.mark.parametrize("arch,tied", [(0, 0), (1, 0), (2, 0), (0, 1), (2, 1)])
def test_finite_differences_every_tensor(arch, tied):
    cfg, theta, tok, lab = _setup(arch, tied=tied)
    loss, g = O.loss_and_grad(cfg, theta, tok, lab)
    rng = np.random.default_rng(0)
    off, h = 0, 1e-5
    for name, shape, _k, _u in O.param_tensors(cfg):
        n = int(np.prod(shape))
        idx = off + rng.choice(n, size=min(n, 6), replace=False)
        if name == "tok_emb":                       # make sure rows that occur are probed
            used = np.unique(tok)[:3]
            idx = np.concatenate([idx, off + used * shape[1] + 1])
        for i in idx:
            tp, tm = theta.copy(), theta.copy()
            tp[i] += h
            tm[i] -= h
            fd = (O.loss_and_grad(cfg, tp, tok, lab, False)[0]
                  - O.loss_and_grad(cfg, tm, tok, lab, False)[0]) / (2 * h)
            assert abs(fd - g[i]) <= 1e-7 + 1e-6 * abs(fd), (name, i - off, fd, g[i])
        off += n


def _torch_forward(cfg, P, tok, lab):
    """Independent forward with torch library routines (float64)."""
    a, L, d, H = cfg["arch"], cfg["n_layers"], cfg["d_model"], cfg["n_heads"]
    B, S = tok.shape
    hd = d // H
    eps = cfg["norm_eps"]
    tok_t = torch.from_numpy(tok.astype(np.int64))

    def rms(x, g):
        return x * torch.rsqrt(x.pow(2).mean(-1, keepdim=True) + eps) * g

    def rope(x):  # x [B,H,S,hd]; complex multiplication form
        i = torch.arange(hd // 2, dtype=torch.float64)
        ang = torch.arange(S, dtype=torch.float64)[:, None] * (cfg["rope_base"] ** (-2 * i / hd))[None]
        z = torch.complex(x[..., : hd // 2], x[..., hd // 2:]) * torch.polar(torch.ones_like(ang), ang)
        return torch.cat([z.real, z.imag], -1)

    def attn(x_in, p):
        qkv = F.linear(x_in, P[p + "wqkv"], P.get(p + "bqkv"))
        q, k, v = [t.reshape(B, S, H, hd).transpose(1, 2) for t in qkv.split(d, dim=-1)]
        if a == 2:
            q, k = rope(q), rope(k)
        c = F.scaled_dot_product_attention(q, k, v, is_causal=(a != 1))
        return F.linear(c.transpose(1, 2).reshape(B, S, d), P[p + "wo"], P.get(p + "bo"))

    x = F.embedding(tok_t, P["tok_emb"])
    if a != 2:
        x = x + P["pos_emb"][:S][None]
    if a == 1:
        x = F.layer_norm(x, (d,), P["lne_g"], P["lne_b"], eps)
    for l in range(L):
        p = f"l{l}."
        if a == 0:
            x = x + attn(F.layer_norm(x, (d,), P[p + "ln1_g"], P[p + "ln1_b"], eps), p)
            h = F.layer_norm(x, (d,), P[p + "ln2_g"], P[p + "ln2_b"], eps)
            x = x + F.linear(F.gelu(F.linear(h, P[p + "w1"], P[p + "b1"])), P[p + "w2"], P[p + "b2"])
        elif a == 1:
            x = F.layer_norm(x + attn(x, p), (d,), P[p + "ln1_g"], P[p + "ln1_b"], eps)
            ff = F.linear(F.gelu(F.linear(x, P[p + "w1"], P[p + "b1"])), P[p + "w2"], P[p + "b2"])
            x = F.layer_norm(x + ff, (d,), P[p + "ln2_g"], P[p + "ln2_b"], eps)
        else:
            x = x + attn(rms(x, P[p + "g1"]), p)
            gu = F.linear(rms(x, P[p + "g2"]), P[p + "wgu"])
            g, u = gu.split(cfg["d_ffn"], dim=-1)
            x = x + F.linear(F.silu(g) * u, P[p + "wd"])
    lab_t = torch.from_numpy(lab.astype(np.int64))
    if a == 1:
        logits = F.linear(x[:, 0, :], P["wc"], P["bc"])
        return F.cross_entropy(logits, lab_t)
    xf = rms(x, P["gf"]) if a == 2 else F.layer_norm(x, (d,), P["lnf_g"], P["lnf_b"], eps)
    logits = F.linear(xf, P["tok_emb"] if cfg.get("tie_embeddings", 0) else P["whead"])
    return F.cross_entropy(logits.reshape(B * S, -1), lab_t.reshape(-1), ignore_index=-1)


@pytest.mark.parametrize("arch,tied", [(0, 0), (1, 0), (2, 0), (0, 1), (2, 1)])
def test_against_torch_autograd(arch, tied):
    cfg, theta, tok, lab = _setup(arch, seed=11, B=3, S=7, tied=tied)
    loss, g = O.loss_and_grad(cfg, theta, tok, lab)
    P, off = {}, 0
    for name, shape, _k, _u in O.param_tensors(cfg):
        n = int(np.prod(shape))
        P[name] = torch.tensor(theta[off:off + n].reshape(shape), dtype=torch.float64, requires_grad=True)
        off += n
    lt = _torch_forward(cfg, P, tok, lab)
    lt.backward()
    assert abs(lt.item() - loss) <= 1e-12 * max(1.0, abs(loss))
    gt = np.concatenate([P[n].grad.numpy().reshape(-1) for n, _s, _k, _u in O.param_tensors(cfg)])
    assert np.max(np.abs(gt - g)) <= 1e-12 * max(1.0, np.max(np.abs(gt)))


def test_tiny_config_c1_against_torch_autograd():
    wl = WORKLOADS["C1"]
    cfg = model_config(wl)
    spec = [(n, s, k) for n, s, k, _u in O.param_tensors(cfg)]
    theta = init_params(5, spec, False).astype(np.float64)
    tok, lab = make_batch(wl, 5, 0)
    loss, g = O.loss_and_grad(cfg, theta, tok, lab)
    assert abs(loss - math.log(256)) < 0.05            # near-uniform prediction at init
    P, off = {}, 0
    for name, shape, _k, _u in O.param_tensors(cfg):
        n = int(np.prod(shape))
        P[name] = torch.tensor(theta[off:off + n].reshape(shape), requires_grad=True)
        off += n
    lt = _torch_forward(cfg, P, tok, lab)
    lt.backward()
    gt = np.concatenate([P[n].grad.numpy().reshape(-1) for n, _s, _k, _u in O.param_tensors(cfg)])
    assert np.max(np.abs(gt - g)) <= 1e-12


@pytest.mark.parametrize("arch", [0, 2])
def test_tied_gradient_is_the_sum_over_both_uses(arch):
    """Chain rule: with the output matrix set equal to the token table, the tied model computes the same
    loss as the untied one, every other gradient is the same, and the table's gradient is the untied
    table's plus the untied output matrix's."""
    cfg_t, theta_t, tok, lab = _setup(arch, seed=7, tied=1)
    cfg_u = dict(cfg_t, tie_embeddings=0)
    V, d = cfg_t["vocab"], cfg_t["d_model"]
    theta_u = np.concatenate([theta_t, theta_t[:V * d]])          # whead is the last tensor of the untied layout
    assert O.param_tensors(cfg_u)[-1][0] == "whead" and O.param_tensors(cfg_u)[0][0] == "tok_emb"
    loss_t, g_t = O.loss_and_grad(cfg_t, theta_t, tok, lab)
    loss_u, g_u = O.loss_and_grad(cfg_u, theta_u, tok, lab)
    assert loss_t == loss_u
    n = theta_t.size
    assert np.array_equal(g_t[V * d:], g_u[V * d:n])
    assert np.max(np.abs(g_t[:V * d] - (g_u[:V * d] + g_u[n:]))) <= 1e-15
    assert O.n_units(cfg_t) == O.n_units(cfg_u) and O.unit_ranges(cfg_t)[-1][1] == O.unit_ranges(cfg_u)[-1][1] - V * d
