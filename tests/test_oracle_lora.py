"""Pins of the oracle's low-rank-adapter step (the LoRA baseline whose step time section 4.3 sets beside HiFT's):
central finite differences of the adapter gradient, an adapter that is a reparametrisation and nothing else (merged
weights give the same loss; a zero B gives the base model), an independent torch-autograd evaluation of the same
low-rank forward, and the AdamW trajectory against torch.optim.AdamW."""
import numpy as np
import pytest

from hift_inputs import init_params, make_batch, model_config
from oracle import hift_oracle as O

SMALL = {
    0: dict(arch=0, n_layers=2, d_model=16, n_heads=2, d_ffn=32, vocab=50, max_seq=12, n_classes=0, norm_eps=1e-5,
            rope_base=10000.0, dtype=0, batch=2, seq=10),
    1: dict(arch=1, n_layers=2, d_model=16, n_heads=2, d_ffn=32, vocab=50, max_seq=12, n_classes=3, norm_eps=1e-5,
            rope_base=10000.0, dtype=0, batch=3, seq=8),
    2: dict(arch=2, n_layers=2, d_model=16, n_heads=2, d_ffn=24, vocab=50, max_seq=12, n_classes=0, norm_eps=1e-5,
            rope_base=10000.0, dtype=0, batch=2, seq=10),
}
RANK, ALPHA = 4, 6.0


def _setup(arch, seed=3):
    wl = SMALL[arch]
    cfg = model_config(wl)
    spec = [(n, s, k) for n, s, k, _u in O.param_tensors(cfg)]
    theta = init_params(seed, spec, False, std=0.3, jitter=0.1).astype(np.float64)
    lora = np.random.default_rng(seed).standard_normal(O.lora_n_params(cfg, RANK)) * 0.2
    tok, lab = make_batch(wl, seed, 1)
    return cfg, theta, lora, tok, lab


@pytest.mark.parametrize("arch", [0, 1, 2])
def test_adapter_gradient_by_central_differences(arch):
    cfg, theta, lora, tok, lab = _setup(arch)
    _loss, g = O.lora_loss_and_grad(cfg, theta, lora, tok, lab, RANK, ALPHA)
    rng = np.random.default_rng(1)
    h = 1e-6
    for i in rng.choice(lora.size, 40, replace=False):
        lp, lm = lora.copy(), lora.copy()
        lp[i] += h
        lm[i] -= h
        fp, _ = O.loss_and_grad(cfg, O.lora_merge(cfg, theta, lp, RANK, ALPHA), tok, lab, need_grad=False)
        fm, _ = O.loss_and_grad(cfg, O.lora_merge(cfg, theta, lm, RANK, ALPHA), tok, lab, need_grad=False)
        fd = (fp - fm) / (2 * h)
        assert abs(fd - g[i]) <= 1e-6 * max(1.0, abs(fd)) + 1e-8, (i, fd, g[i])


def test_zero_b_is_the_base_model_and_only_b_has_a_gradient():
    cfg, theta, lora, tok, lab = _setup(2)
    V = O._lora_views(cfg, RANK, lora)
    for name in V:
        if "lora_b" in name:
            V[name][...] = 0.0
    loss, g = O.lora_loss_and_grad(cfg, theta, lora, tok, lab, RANK, ALPHA)
    base, _ = O.loss_and_grad(cfg, theta, tok, lab, need_grad=False)
    assert loss == base
    G = O._lora_views(cfg, RANK, g)
    assert all(np.all(G[n] == 0) for n in G if "lora_a" in n)          # d loss / d A = s B^T G = 0
    assert all(np.any(G[n] != 0) for n in G if "lora_b" in n)


def test_low_rank_forward_written_with_torch_gives_the_same_gradient():
    """The same adapters as an explicit second path q = x Wq^T + s (x Aq^T) Bq^T through torch autograd: what the
    GPU path computes, against the oracle's merged-weight definition."""
    import torch
    cfg, theta, lora, tok, lab = _setup(2)
    d, H, L, r, s = cfg["d_model"], cfg["n_heads"], cfg["n_layers"], RANK, ALPHA / RANK
    hd = d // H
    P = {k: torch.tensor(v.copy()) for k, v in O._Params(cfg, theta).views.items()}
    A = {k: torch.tensor(v.copy(), requires_grad=True) for k, v in O._lora_views(cfg, RANK, lora).items()}
    B_, S = tok.shape
    pos = torch.arange(S, dtype=torch.float64)
    inv = cfg["rope_base"] ** (-torch.arange(0, hd // 2, dtype=torch.float64) * 2.0 / hd)
    ang = pos[:, None] * inv[None, :]
    cos, sin = torch.cos(ang), torch.sin(ang)

    def rope(x):                                   # [B, H, S, hd], pairs (i, i + hd/2)
        x1, x2 = x[..., :hd // 2], x[..., hd // 2:]
        return torch.cat([x1 * cos - x2 * sin, x2 * cos + x1 * sin], -1)

    def rms(x, g):
        return x / torch.sqrt((x * x).mean(-1, keepdim=True) + cfg["norm_eps"]) * g

    x = P["tok_emb"][torch.tensor(tok.astype(np.int64))]           # [B, S, d]
    for l in range(L):
        p = f"l{l}."
        h = rms(x, P[p + "g1"])
        qkv = h @ P[p + "wqkv"].T
        q = qkv[..., :d] + s * (h @ A[p + "lora_aq"].T) @ A[p + "lora_bq"].T
        k = qkv[..., d:2 * d]
        v = qkv[..., 2 * d:] + s * (h @ A[p + "lora_av"].T) @ A[p + "lora_bv"].T
        sp = lambda t: t.reshape(B_, S, H, hd).transpose(1, 2)
        q, k, v = rope(sp(q)), rope(sp(k)), sp(v)
        sc = q @ k.transpose(-1, -2) / np.sqrt(hd)
        sc = sc.masked_fill(torch.triu(torch.ones(S, S, dtype=torch.bool), 1), float("-inf"))
        ctx = (torch.softmax(sc, -1) @ v).transpose(1, 2).reshape(B_, S, d)
        x = x + ctx @ P[p + "wo"].T
        h2 = rms(x, P[p + "g2"])
        gu = h2 @ P[p + "wgu"].T
        f = gu.shape[-1] // 2
        x = x + (torch.nn.functional.silu(gu[..., :f]) * gu[..., f:]) @ P[p + "wd"].T
    logits = rms(x, P["gf"]) @ P["whead"].T
    loss = torch.nn.functional.cross_entropy(logits.reshape(-1, logits.shape[-1]), torch.tensor(lab.astype(np.int64)).reshape(-1),
                                            ignore_index=-1)
    loss.backward()
    lo, g = O.lora_loss_and_grad(cfg, theta, lora, tok, lab, RANK, ALPHA)
    assert abs(loss.item() - lo) <= 1e-12 * abs(lo)
    G = O._lora_views(cfg, RANK, g)
    for name in G:
        assert np.allclose(A[name].grad.numpy(), G[name], rtol=1e-9, atol=1e-13), name


def test_adapter_training_follows_adamw_and_leaves_the_base_untouched():
    import torch
    cfg, theta, lora, tok, lab = _setup(0)
    opt = dict(kind="adamw", lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.05)
    orc = O.LoraOracle(cfg, opt, theta, lora, RANK, ALPHA)
    p = torch.nn.Parameter(torch.tensor(lora.copy()))
    topt = torch.optim.AdamW([p], lr=opt["lr"], betas=(0.9, 0.999), eps=1e-8, weight_decay=0.05)
    for t in range(1, 4):
        tok, lab = make_batch(SMALL[0], 3, t)
        _l, g = O.lora_loss_and_grad(cfg, theta, p.detach().numpy().copy(), tok, lab, RANK, ALPHA)
        p.grad = torch.tensor(g)
        topt.step()
        orc.step(tok, lab)
        assert np.allclose(orc.lora, p.detach().numpy(), rtol=1e-12, atol=1e-15), t
    assert np.array_equal(orc.theta, theta)
