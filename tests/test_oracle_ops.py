"""Textbook special cases of the oracle's building blocks."""
import math

import numpy as np

from oracle import hift_oracle as O

R = np.random.default_rng(0)


def test_softmax_rows_sum_to_one_and_shift_invariant():
    s = R.standard_normal((5, 9)) * 10
    p = O.softmax_lastdim(s)
    assert np.allclose(p.sum(-1), 1.0, atol=1e-15)
    assert np.allclose(p, O.softmax_lastdim(s + 1000.0), atol=1e-13)


def test_cross_entropy_uniform_logits_is_log_vocab():
    loss, dl = O.cross_entropy_fwd(np.zeros((6, 50)), np.array([3, 1, -1, 49, 0, -1]))
    assert abs(loss - math.log(50)) < 1e-14
    assert np.all(dl[2] == 0) and np.all(dl[5] == 0)
    assert np.allclose(dl.sum(-1), 0, atol=1e-16)
    assert np.isclose(dl[0, 3], (1 / 50 - 1) / 4)


def test_cross_entropy_without_a_single_target_is_zero():
    """The empty mean is read as the empty sum: loss 0, no gradient (sequences of one token have no next token)."""
    loss, dl = O.cross_entropy_fwd(np.random.default_rng(0).standard_normal((4, 9)), np.full(4, -1))
    assert loss == 0.0 and dl.shape == (4, 9) and not dl.any()
    # and a decoder step on one-token sequences moves nothing
    cfg = dict(arch=0, n_layers=1, d_model=8, n_heads=2, d_ffn=16, vocab=11, max_seq=4, n_classes=0, norm_eps=1e-5,
               rope_base=10000.0, dtype=0)
    n = sum(int(np.prod(sh)) for _n, sh, _k, _u in O.param_tensors(cfg))
    theta = np.random.default_rng(1).standard_normal(n) * 0.1
    tok = np.array([[3], [7]], np.int32)
    loss, g = O.loss_and_grad(cfg, theta, tok, np.full((2, 1), -1, np.int32))
    assert loss == 0.0 and not g.any()


def test_rope_is_a_rotation():
    x = R.standard_normal((2, 3, 7, 8))
    cos, sin = O.rope_angles(7, 8, 10000.0, np.float64)
    y = O.rope_fwd(x, cos, sin)
    assert np.allclose(x[..., :4] ** 2 + x[..., 4:] ** 2, y[..., :4] ** 2 + y[..., 4:] ** 2)
    assert np.allclose(y[:, :, 0], x[:, :, 0])                 # position 0: angle 0
    assert np.allclose(O.rope_bwd(y, cos, sin), x)             # adjoint = inverse rotation
    # pair 0 at position p turns by exactly p radians
    assert np.isclose(y[0, 0, 3, 0], x[0, 0, 3, 0] * math.cos(3) - x[0, 0, 3, 4] * math.sin(3))


def test_rope_scores_depend_on_relative_position_only():
    q, k = R.standard_normal(8), R.standard_normal(8)
    cos, sin = O.rope_angles(12, 8, 10000.0, np.float64)
    qq = np.broadcast_to(q, (1, 1, 12, 8))
    kk = np.broadcast_to(k, (1, 1, 12, 8))
    s = O.rope_fwd(qq, cos, sin)[0, 0] @ O.rope_fwd(kk, cos, sin)[0, 0].T
    assert np.allclose(s[5, 2], s[9, 6]) and np.allclose(s[3, 3], q @ k)


def test_norms():
    x = R.standard_normal((4, 32)) * 3 + 1
    y, _ = O.layernorm_fwd(x, np.ones(32), np.zeros(32), 0.0)
    assert np.allclose(y.mean(-1), 0, atol=1e-14) and np.allclose(y.var(-1), 1, atol=1e-12)
    y, _ = O.rmsnorm_fwd(x, np.ones(32), 0.0)
    assert np.allclose((y * y).mean(-1), 1, atol=1e-12)


def test_attention_special_cases():
    q, k, v = (R.standard_normal((1, 2, 5, 4)) for _ in range(3))
    ctx, p = O.attention_fwd(q, k, v, True)
    assert np.allclose(ctx[:, :, 0], v[:, :, 0])               # first causal row sees one key
    assert np.allclose(np.triu(p[0, 0], 1), 0)
    ctx, p = O.attention_fwd(np.zeros_like(q), k, v, False)     # zero queries: plain average
    assert np.allclose(ctx, np.broadcast_to(v.mean(2, keepdims=True), v.shape))
    ctx1, _ = O.attention_fwd(q[:, :, :1], k[:, :, :1], v[:, :, :1], False)
    assert np.allclose(ctx1, v[:, :, :1])                      # one token: output = V


def test_gelu_and_silu_values():
    assert np.isclose(O.gelu_fwd(np.array([0.0, 1.0]))[1], 0.8413447460685429)   # Phi(1)
    assert np.isclose(O.silu(np.array([1.0]))[0], 1 / (1 + math.exp(-1)))
    assert np.isclose(O.gelu_bwd(np.ones(1), np.zeros(1))[0], 0.5)
