"""GPU parity of single kernels through the C ABI: the contraction in every operand layout
(bf16 MFMA path and fp32 path), the optimizer update, normalisation and cross-entropy.
Expected values: the plain definitions in float64 (numpy matmul; the oracle's own functions)."""
import numpy as np
import pytest

from oracle import hift_oracle as O

pytestmark = pytest.mark.gpu

F32, BF16 = 0, 1


def _bf16_round(x):
    from hift_inputs import round_to_bf16
    return round_to_bf16(x.astype(np.float32))


def _dev(x, bf16):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if bf16 else t


CASES = [  # M, N, K  (several tiles + ragged tails; K not a multiple of 64; tiny)
    (256, 256, 64), (512, 768, 256), (384, 640, 192), (136, 72, 40), (1000, 264, 520), (8, 3, 64), (64, 64, 8),
    (2048, 512, 128), (300, 200, 100),
    # enough 256x256 tiles to take the large-tile kernels (k-major pair: the direct-to-LDS kernel)
    (2048, 8192, 96), (2000, 8200, 160), (1800, 7944, 64),
]


@pytest.mark.parametrize("dtype", [F32, BF16], ids=["f32", "bf16"])
@pytest.mark.parametrize("ak,bk", [(1, 1), (1, 0), (0, 1), (0, 0)])
@pytest.mark.parametrize("M,N,K", CASES)
def test_gemm_layouts(dtype, ak, bk, M, N, K):
    import torch
    import paper_2401_15207_amd as H
    rng = np.random.default_rng(M * 7 + N * 3 + K + ak * 2 + bk)
    bf = dtype == BF16
    A = rng.standard_normal((M, K)).astype(np.float32)
    B = rng.standard_normal((N, K)).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    R = rng.standard_normal((M, N)).astype(np.float32)
    if bf:
        A, B, bias, R = map(_bf16_round, (A, B, bias, R))
    ref = A.astype(np.float64) @ B.astype(np.float64).T + bias + R
    dA = _dev(A if ak else A.T, bf)
    dB = _dev(B if bk else B.T, bf)
    lda = K if ak else M
    ldb = K if bk else N
    for out_f32 in ([1] if not bf else [0, 1]):
        dC = torch.zeros((M, N), dtype=torch.float32 if out_f32 else torch.bfloat16, device="cuda")
        dR = _dev(R, bf and not out_f32)
        H.kernel_gemm(dtype, ak, bk, out_f32, M, N, K, dA, lda, dB, ldb, dC, N, _dev(bias, bf), dR)
        torch.cuda.synchronize()
        got = dC.float().cpu().numpy().astype(np.float64)
        scale = np.sqrt(K) + 1.0
        if bf and not out_f32:
            tol = 2 ** -8 * (np.abs(ref) + 0.02 * scale)    # one bf16 rounding of the result
        elif bf:
            tol = 1e-5 * (np.abs(ref) + scale)               # exact products, fp32 accumulation
        else:
            tol = 2e-6 * (np.abs(ref) + scale)
        bad = np.abs(got - ref) > tol
        assert not bad.any(), (out_f32, int(bad.sum()), float(np.max(np.abs(got - ref))))


@pytest.mark.parametrize("M,N,K", [(4096, 4096, 2048), (12288, 4096, 512), (8192, 2816, 96), (5632, 4096, 32), (32000, 4096, 64)])
def test_weight_gradient_contraction(M, N, K):
    """dW = dY^T . X with both operands stored contraction-index first (the layout the backward pass leaves them in), at
    shapes the direct-to-LDS / transposing-read kernel takes (M and N multiples of 256, K of 32): fp32 and bf16 output,
    with and without bias and residual, against the float64 product."""
    import torch
    import paper_2401_15207_amd as H
    rng = np.random.default_rng(M + N + K)
    A = _bf16_round(rng.standard_normal((K, M)))          # [k][m]
    B = _bf16_round(rng.standard_normal((K, N)))          # [k][n]
    bias = _bf16_round(rng.standard_normal(N))
    ref0 = A.astype(np.float64).T @ B.astype(np.float64)
    dA, dB = _dev(A, True), _dev(B, True)
    for out_f32, extras in ((1, False), (0, True), (1, True)):
        R = rng.standard_normal((M, N)).astype(np.float32)
        if not out_f32:
            R = _bf16_round(R)
        ref = ref0 + (bias + R if extras else 0.0)
        dC = torch.full((M, N), float("nan"), dtype=torch.float32 if out_f32 else torch.bfloat16, device="cuda")
        H.kernel_gemm(BF16, 0, 0, out_f32, M, N, K, dA, M, dB, N, dC, N, _dev(bias, True) if extras else None,
                      _dev(R, not out_f32) if extras else None)
        torch.cuda.synchronize()
        got = dC.float().cpu().numpy().astype(np.float64)
        scale = np.sqrt(K) + 1.0
        tol = (1e-5 * (np.abs(ref) + scale)) if out_f32 else 2 ** -8 * (np.abs(ref) + 0.02 * scale)
        bad = np.abs(got - ref) > tol
        assert not bad.any(), (out_f32, extras, int(bad.sum()), float(np.max(np.abs(got - ref))))


def test_gemm_batched_strided_bf16():
    import torch
    import paper_2401_15207_amd as H
    rng = np.random.default_rng(0)
    nb, M, N, K = 6, 128, 192, 64
    A = _bf16_round(rng.standard_normal((nb, M, K)))
    B = _bf16_round(rng.standard_normal((nb, N, K)))
    dA, dB = _dev(A, True), _dev(B, True)
    dC = torch.zeros((nb, M, N), dtype=torch.bfloat16, device="cuda")
    H.kernel_gemm(BF16, 1, 1, 0, M, N, K, dA, K, dB, K, dC, N, None, None, batch=nb, sa=M * K, sb=N * K, sc=M * N)
    torch.cuda.synchronize()
    ref = np.einsum("bmk,bnk->bmn", A.astype(np.float64), B.astype(np.float64))
    got = dC.float().cpu().numpy()
    assert np.all(np.abs(got - ref) <= 2 ** -8 * (np.abs(ref) + 0.2))


@pytest.mark.parametrize("bk", [1, 0], ids=["w_kmajor", "w_transposed"])
@pytest.mark.parametrize("M,N,K", [(2048, 8192, 96), (2000, 8200, 160), (1800, 7944, 64), (2048, 12288, 4096),
                                   (2048, 4096, 352), (1990, 3592, 96),
                                   # more column tiles than compute units twice over; a short and ragged M with many columns
                                   (2048, 8192, 192), (1000, 16128, 128), (2048, 22016, 256)])
def test_gemm_with_packed_weight_operand(M, N, K, bk):
    import torch
    import paper_2401_15207_amd as H
    rng = np.random.default_rng(M + N + K + bk)
    A = _bf16_round(rng.standard_normal((M, K)))
    B = _bf16_round(rng.standard_normal((N, K)) * 0.5)
    bias = _bf16_round(rng.standard_normal(N))
    R = _bf16_round(rng.standard_normal((M, N)))
    ref = A.astype(np.float64) @ B.astype(np.float64).T + bias + R
    nbytes = H.kernel_packed_bytes(N, K)
    assert nbytes == ((N + 255) // 256) * 256 * K * 2
    dBp = torch.full((nbytes // 2,), float("nan"), dtype=torch.bfloat16, device="cuda")   # every block must be written
    dB = _dev(B if bk else B.T, True)
    H.kernel_pack_b(bk, N, K, dB, K if bk else N, dBp)
    dA = _dev(A, True)
    for out_f32 in (0, 1):
        dC = torch.zeros((M, N), dtype=torch.float32 if out_f32 else torch.bfloat16, device="cuda")
        H.kernel_gemm_packed(out_f32, M, N, K, dA, K, dBp, dC, N, _dev(bias, True), _dev(R, not out_f32))
        torch.cuda.synchronize()
        got = dC.float().cpu().numpy().astype(np.float64)
        scale = np.sqrt(K) + 1.0
        tol = (1e-5 if out_f32 else 2 ** -8) * (np.abs(ref) + (scale if out_f32 else 0.02 * scale))
        bad = np.abs(got - ref) > tol
        assert not bad.any(), (out_f32, int(bad.sum()), float(np.max(np.abs(got - ref))))


@pytest.mark.parametrize("bk", [1, 0], ids=["w_kmajor", "w_transposed"])
def test_pack_of_unaligned_source_matches_aligned(bk):
    """The fragment-order copy is a pure permutation (plus zero rows up to a multiple of 256): the
    packer for sources without 16-byte alignment must write the same bytes as the tiled one."""
    import torch
    import paper_2401_15207_amd as H
    N, K = 1000, 96
    rng = np.random.default_rng(bk)
    B = _bf16_round(rng.standard_normal((N, K)))
    src = B if bk else B.T
    rows, cols = src.shape
    nbytes = H.kernel_packed_bytes(N, K)
    p1 = torch.full((nbytes // 2,), float("nan"), dtype=torch.bfloat16, device="cuda")
    p2 = torch.full((nbytes // 2,), float("nan"), dtype=torch.bfloat16, device="cuda")
    H.kernel_pack_b(bk, N, K, _dev(src, True), cols, p1)
    wide = torch.zeros((rows, cols + 3), dtype=torch.bfloat16, device="cuda")   # odd leading dimension
    wide[:, :cols] = _dev(src, True)
    H.kernel_pack_b(bk, N, K, wide, cols + 3, p2)
    torch.cuda.synchronize()
    a, b = p1.view(torch.int16).cpu().numpy(), p2.view(torch.int16).cpu().numpy()
    assert np.array_equal(a, b)
    # block (nb, kk), lane l, element e  <-  B[nb*32 + pi(l%32)][kk*16 + (l/32)*8 + e], pi = bits 2 and 3 exchanged
    blk = a.view(np.uint16).reshape(-1, K // 16, 64, 8)
    want = np.zeros((blk.shape[0] * 32, K), np.float32)
    want[:N] = B
    r = np.arange(32)
    pi = (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1)
    want = want.reshape(-1, 32, K)[:, pi, :]
    want = want.reshape(-1, 32, K // 16, 2, 8).transpose(0, 2, 3, 1, 4).reshape(blk.shape)
    assert np.array_equal((blk.astype(np.uint32) << 16).view(np.float32), want)


def test_gemm_empty():
    import torch
    import paper_2401_15207_amd as H
    z = torch.zeros(8, device="cuda")
    H.kernel_gemm(F32, 1, 1, 1, 0, 4, 4, z, 4, z, 4, z, 4)
    H.kernel_gemm(F32, 1, 1, 1, 2, 2, 0, z, 0, z, 0, z, 2)   # K = 0: result is zero (+0)
    torch.cuda.synchronize()
    assert float(z[:4].abs().sum()) == 0.0


def test_leading_dimension_shorter_than_a_row_is_refused():
    """The kernels would read past the operand: the entry points turn the call down instead."""
    import torch
    import paper_2401_15207_amd as H
    z = torch.zeros(16, device="cuda")
    for lda, ldb, ldc in [(3, 4, 4), (4, 3, 4), (4, 4, 3)]:
        with pytest.raises(H.HiftError):
            H.kernel_gemm(F32, 1, 1, 1, 4, 4, 4, z, lda, z, ldb, z, ldc)
    big = torch.zeros(512 * 64, device="cuda", dtype=torch.bfloat16)
    packed = torch.zeros(H.kernel_packed_bytes(256, 64), device="cuda", dtype=torch.uint8)
    with pytest.raises(H.HiftError):
        H.kernel_pack_b(1, 256, 64, big, 32, packed)    # B(n,k) at B[n*ldb + k] needs ldb >= K
    with pytest.raises(H.HiftError):
        H.kernel_pack_b(0, 256, 64, big, 64, packed)    # B(n,k) at B[k*ldb + n] needs ldb >= N


@pytest.mark.parametrize("kind", ["adamw", "adagrad", "sgdm", "sgd"])
@pytest.mark.parametrize("n", [1, 7, 4096, 100003])
def test_optimizer_kernel_against_oracle_formulas(kind, n):
    import torch
    import paper_2401_15207_amd as H
    rng = np.random.default_rng(n)
    opt = {"adamw": dict(kind="adamw", lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, momentum=0.0),
           "adagrad": dict(kind="adagrad", lr=1e-2, beta1=0, beta2=0, eps=1e-10, weight_decay=0.0, momentum=0.0),
           "sgdm": dict(kind="sgd", lr=1e-2, beta1=0, beta2=0, eps=0, weight_decay=0.0, momentum=0.9),
           "sgd": dict(kind="sgd", lr=1e-2, beta1=0, beta2=0, eps=0, weight_decay=0.001, momentum=0.0)}[kind]
    th = rng.standard_normal(n).astype(np.float32)
    s1, s2 = np.zeros(n, np.float32), np.zeros(n, np.float32)
    d_th, d_s1, d_s2 = (torch.from_numpy(x.copy()).cuda() for x in (th, s1, s2))
    d_cc = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    o_th, o_s1, o_s2 = th.astype(np.float64), s1.astype(np.float64), s2.astype(np.float64)
    dm = np.ones(n)
    for t in (1, 2, 3):
        g = (rng.standard_normal(n) * 0.1).astype(np.float32)
        H.kernel_optimizer(opt, n, 1, t, d_th, torch.from_numpy(g).cuda(), d_s1, d_s2, d_cc)
        torch.cuda.synchronize()
        if opt["kind"] == "adamw":
            O.adamw_update(o_th, g.astype(np.float64), o_s1, o_s2, t, opt["lr"], opt["beta1"], opt["beta2"], opt["eps"], opt["weight_decay"], dm)
        elif opt["kind"] == "adagrad":
            O.adagrad_update(o_th, g.astype(np.float64), o_s1, opt["lr"], opt["eps"], opt["weight_decay"], dm)
        else:
            O.sgd_update(o_th, g.astype(np.float64), o_s1, t, opt["lr"], opt["momentum"], opt["weight_decay"], dm)
        got = d_th.cpu().numpy()
        assert np.all(np.abs(got - o_th) <= 4e-7 * np.abs(o_th) + 1e-5 * opt["lr"]), t   # fp32 storage of theta, t roundings
        cc = d_cc.float().cpu().numpy()
        assert np.array_equal(cc, _bf16_round(got))          # bf16 copy = round-to-nearest-even of the master
    if kind in ("adamw", "adagrad", "sgdm"):
        assert np.allclose(d_s1.cpu().numpy(), o_s1, rtol=1e-5, atol=1e-7)   # sums of both signs cancel
    if kind == "adamw":
        assert np.allclose(d_s2.cpu().numpy(), o_s2, rtol=1e-5, atol=1e-12)


@pytest.mark.parametrize("dtype", [F32, BF16], ids=["f32", "bf16"])
@pytest.mark.parametrize("rows,d", [(5, 64), (1, 8), (130, 4096), (3, 100), (0, 64)])
@pytest.mark.parametrize("rms", [0, 1])
def test_norm_forward(dtype, rows, d, rms):
    import torch
    import paper_2401_15207_amd as H
    rng = np.random.default_rng(rows + d)
    bf = dtype == BF16
    x = (rng.standard_normal((rows, d)) * 2 + 0.5).astype(np.float32)
    g = (1 + 0.1 * rng.standard_normal(d)).astype(np.float32)
    b = (0.1 * rng.standard_normal(d)).astype(np.float32)
    if bf:
        x, g, b = map(_bf16_round, (x, g, b))
    dy = torch.zeros((rows, d), dtype=torch.bfloat16 if bf else torch.float32, device="cuda")
    st = torch.zeros((max(rows, 1), 2), device="cuda")
    H.kernel_norm_fwd(dtype, rms, rows, d, 1e-5, _dev(x, bf), _dev(g, bf), _dev(b, bf), dy, st)
    torch.cuda.synchronize()
    if rows == 0:
        return
    X = x.astype(np.float64)
    ref, (_xh, rstd) = (O.rmsnorm_fwd(X, g.astype(np.float64), 1e-5) if rms
                        else O.layernorm_fwd(X, g.astype(np.float64), b.astype(np.float64), 1e-5))
    got = dy.float().cpu().numpy()
    tol = (2 ** -8 if bf else 3e-6) * (np.abs(ref) + (1e-2 if bf else 1.0))   # fp32: terms of size 1 may cancel
    assert np.all(np.abs(got - ref) <= tol)
    assert np.allclose(st[:rows, 1].cpu().numpy(), rstd[:, 0], rtol=2e-6)


@pytest.mark.parametrize("dtype", [F32, BF16], ids=["f32", "bf16"])
@pytest.mark.parametrize("rows,V", [(7, 256), (64, 32000), (5, 3), (1, 2), (0, 16), (9, 50272), (3, 16392), (5, 65544), (300, 32000)])
def test_cross_entropy(dtype, rows, V):
    import torch
    import paper_2401_15207_amd as H
    rng = np.random.default_rng(rows * 31 + V)
    bf = dtype == BF16
    z = (rng.standard_normal((rows, V)) * 3).astype(np.float32)
    if bf:
        z = _bf16_round(z)
    lab = rng.integers(0, V, size=rows).astype(np.int32)
    if rows > 2:
        lab[1] = -1
    dz = _dev(z, bf)
    scratch = torch.zeros(rows + 1, device="cuda")
    loss = torch.full((1,), -7.0, device="cuda")
    H.kernel_cross_entropy(dtype, rows, V, dz, torch.from_numpy(lab).cuda(), scratch, loss)
    torch.cuda.synchronize()
    if rows == 0:
        assert float(loss) == 0.0
        return
    ref_loss, ref_d = O.cross_entropy_fwd(z.astype(np.float64), lab.astype(np.int64))
    assert abs(float(loss) - ref_loss) <= 2e-6 * abs(ref_loss) + 1e-6
    got = dz.float().cpu().numpy()
    tol = (2 ** -8 if bf else 1e-5) * np.abs(ref_d) + 1e-8
    assert np.all(np.abs(got - ref_d) <= tol)


@pytest.mark.parametrize("dtype", [F32, BF16], ids=["f32", "bf16"])
def test_cross_entropy_without_any_target(dtype):
    # no row has a label: the loss is 0 (not 0 / 0) and every gradient is zero
    import torch
    import paper_2401_15207_amd as H
    rows, V = 6, 1000
    z = np.random.default_rng(1).standard_normal((rows, V)).astype(np.float32)
    dz = _dev(z, dtype == BF16)
    scratch = torch.zeros(rows + 1, device="cuda")
    loss = torch.full((1,), -7.0, device="cuda")
    H.kernel_cross_entropy(dtype, rows, V, dz, torch.full((rows,), -1, dtype=torch.int32, device="cuda"), scratch, loss)
    torch.cuda.synchronize()
    assert float(loss) == 0.0 and float(dz.float().abs().max()) == 0.0


def test_fused_attention_refuses_what_it_cannot_take():
    import torch
    import paper_2401_15207_amd as H_
    z = torch.zeros(77 * 3 * 64 * 2, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(H_.HiftError):            # rows of the probability matrix must be multiples of 16 bytes
        H_.kernel_attention_fwd(1, 2, 77, 64, 1, z, z, z)
    with pytest.raises(H_.HiftError):            # head widths 64 and 128 only
        H_.kernel_attention_fwd(1, 2, 64, 32, 1, z, z, z)


@pytest.mark.parametrize("B,H,S,hd,causal", [(2, 3, 200, 64, 1), (1, 2, 512, 128, 1), (2, 2, 136, 128, 0), (1, 2, 72, 64, 1),
                                              (1, 1, 8, 128, 1), (2, 4, 384, 64, 0)])
def test_fused_attention_forward(B, H, S, hd, causal):
    """Scores, softmax and P.V in one kernel against the oracle's attention (float64).  Probabilities
    and context are bf16: 2^-8 relative plus the rounding of inputs that are sums of S terms."""
    import torch
    import paper_2401_15207_amd as H_
    from oracle import hift_oracle as O
    rng = np.random.default_rng(B * 1000 + S + hd + causal)
    d = H * hd
    qkv = _bf16_round(rng.standard_normal((B * S, 3 * d)) * 1.5)
    q = qkv[:, :d].reshape(B, S, H, hd).transpose(0, 2, 1, 3).astype(np.float64)
    k = qkv[:, d:2 * d].reshape(B, S, H, hd).transpose(0, 2, 1, 3).astype(np.float64)
    v = qkv[:, 2 * d:].reshape(B, S, H, hd).transpose(0, 2, 1, 3).astype(np.float64)
    ctx_ref, p_ref = O.attention_fwd(q, k, v, bool(causal))
    dq = _dev(qkv, True)
    dp = torch.full((B, H, S, S), float("nan"), dtype=torch.bfloat16, device="cuda")   # every entry must be written
    dc = torch.full((B * S, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    dl = torch.full((B * H * S,), float("nan"), dtype=torch.float32, device="cuda")
    H_.kernel_attention_fwd(B, H, S, hd, causal, dq, dp, dc, dl)
    torch.cuda.synchronize()
    # log2 of each row's sum of exponentials, against the library's log-sum-exp of the masked scaled scores
    from scipy.special import logsumexp
    sc = np.matmul(q, np.swapaxes(k, -1, -2)) / np.sqrt(hd)
    if causal:
        sc = np.where(np.tril(np.ones((S, S), bool)), sc, -np.inf)
    lse_ref = logsumexp(sc, axis=-1) / np.log(2.0)
    assert np.all(np.abs(dl.cpu().numpy().reshape(B, H, S) - lse_ref) <= 2e-5 * np.abs(lse_ref) + 2e-5)
    # without the probabilities (one pass, normalised at the end): the same context and log-sums to the same bars
    dc2 = torch.full((B * S, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    dl2 = torch.full((B * H * S,), float("nan"), dtype=torch.float32, device="cuda")
    H_.kernel_attention_fwd(B, H, S, hd, causal, dq, None, dc2, dl2)
    torch.cuda.synchronize()
    assert np.all(np.abs(dl2.cpu().numpy().reshape(B, H, S) - lse_ref) <= 2e-5 * np.abs(lse_ref) + 2e-5)
    c2 = dc2.float().cpu().numpy().astype(np.float64).reshape(B, S, H, hd).transpose(0, 2, 1, 3)
    assert np.isfinite(c2).all()
    assert np.all(np.abs(c2 - ctx_ref) <= 2 ** -7 * np.abs(ctx_ref) + 2e-2)
    assert np.sqrt(np.mean((c2 - ctx_ref) ** 2)) <= 4e-3 * np.sqrt(np.mean(ctx_ref ** 2)) + 1e-4
    p = dp.float().cpu().numpy().astype(np.float64)
    c = dc.float().cpu().numpy().astype(np.float64).reshape(B, S, H, hd).transpose(0, 2, 1, 3)
    assert np.isfinite(p).all() and np.isfinite(c).all()
    if causal:
        assert np.all(p[:, :, np.triu_indices(S, 1)[0], np.triu_indices(S, 1)[1]] == 0.0)
    assert np.all(np.abs(p - p_ref) <= 2 ** -8 * p_ref + 1e-6)
    assert np.all(np.abs(p.sum(-1) - 1.0) <= 2e-2)
    assert np.all(np.abs(c - ctx_ref) <= 2 ** -7 * np.abs(ctx_ref) + 2e-2)
    assert np.sqrt(np.mean((c - ctx_ref) ** 2)) <= 4e-3 * np.sqrt(np.mean(ctx_ref ** 2)) + 1e-4


@pytest.mark.parametrize("M,f,K,keep", [(2048, 1664, 256, 1), (1992, 1792, 96, 1), (2048, 11008, 128, 0)])
def test_linear_with_gated_activation_in_the_epilogue(M, f, K, keep):
    """x . [Wg | Wu]^T with silu(gate) * up formed in the contraction's epilogue, against the oracle's
    swiglu on the float64 product.  The activation is computed from the bf16-rounded pre-activations
    (what the backward pass reads), so it is compared with the oracle's function of those."""
    import torch
    import paper_2401_15207_amd as H_
    from oracle import hift_oracle as O
    rng = np.random.default_rng(M + f + K)
    x = _bf16_round(rng.standard_normal((M, K)))
    w = _bf16_round(rng.standard_normal((2 * f, K)) * (1.5 / np.sqrt(K)))
    pre_ref = x.astype(np.float64) @ w.astype(np.float64).T
    dx, dw = _dev(x, True), _dev(w, True)
    scratch = torch.empty(H_.kernel_packed_bytes(2 * f, K) // 2, dtype=torch.bfloat16, device="cuda")
    pre = torch.full((M, 2 * f), float("nan"), dtype=torch.bfloat16, device="cuda")
    act = torch.full((M, f), float("nan"), dtype=torch.bfloat16, device="cuda")
    H_.kernel_linear_fused(H_.EPILOGUE_SWIGLU, M, 2 * f, K, dx, K, dw, scratch, pre if keep else None, act, None, 0, 0)
    torch.cuda.synchronize()
    a = act.float().cpu().numpy().astype(np.float64)
    if keep:
        p = pre.float().cpu().numpy().astype(np.float64)
        assert np.all(np.abs(p - pre_ref) <= 2 ** -8 * np.abs(pre_ref) + 1e-5)
    else:
        assert torch.isnan(pre.float()).all()
        p = _bf16_round(pre_ref).astype(np.float64)      # within one rounding of what the kernel held
    a_ref = O.swiglu_fwd(p[:, :f], p[:, f:])
    if keep:
        assert np.all(np.abs(a - a_ref) <= 2 ** -8 * np.abs(a_ref) + 1e-6)
    else:
        # the kernel's pre-activations may sit one bf16 step from the rounded float64 product
        g, u = p[:, :f], p[:, f:]
        slack = 2 ** -7 * (np.abs(a_ref) + np.abs(u) * (np.abs(g) + 1.0))
        assert np.all(np.abs(a - a_ref) <= slack + 1e-6)


@pytest.mark.parametrize("M,S,heads,K,rot_heads", [(2048, 512, 10, 256, 20), (1000, 200, 18, 96, 24), (2048, 128, 10, 64, 0), (1024, 256, 42, 64, 84)])
def test_linear_with_rotary_embedding_in_the_epilogue(M, S, heads, K, rot_heads):
    """x . Wqkv^T with the rotation of the q and k heads applied to the fp32 accumulators, against the
    oracle's rope on the float64 product (one rounding: 2^-8 relative on the pair's magnitude)."""
    import torch
    import paper_2401_15207_amd as H_
    from oracle import hift_oracle as O
    hd, d = 128, heads * 128
    N = 3 * d
    rng = np.random.default_rng(M + S + heads + K)
    x = _bf16_round(rng.standard_normal((M, K)))
    w = _bf16_round(rng.standard_normal((N, K)) / np.sqrt(K))
    y_ref = x.astype(np.float64) @ w.astype(np.float64).T
    cos, sin = O.rope_angles(S, hd, 10000.0, np.float64)
    pos = np.arange(M) % S
    rot_cols = rot_heads * hd
    blk = y_ref[:, :rot_cols].reshape(M, rot_heads, hd).transpose(1, 0, 2)           # [heads, M, hd]
    if rot_heads:
        y_ref[:, :rot_cols] = O.rope_fwd(blk, cos[pos], sin[pos]).transpose(1, 0, 2).reshape(M, rot_cols)
    mag = np.abs(y_ref).copy()
    if rot_heads:
        pair = np.abs(blk) + np.abs(np.roll(blk, hd // 2, axis=-1))
        mag[:, :rot_cols] = pair.transpose(1, 0, 2).reshape(M, rot_cols)
    tab = torch.from_numpy(np.stack([cos, sin], -1).astype(np.float32)).cuda().contiguous()
    scratch = torch.empty(H_.kernel_packed_bytes(N, K) // 2, dtype=torch.bfloat16, device="cuda")
    y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    H_.kernel_linear_fused(H_.EPILOGUE_ROPE, M, N, K, _dev(x, True), K, _dev(w, True), scratch, y, None, tab, S, rot_cols)
    torch.cuda.synchronize()
    got = y.float().cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - y_ref) <= 2 ** -8 * np.abs(y_ref) + 1e-5 * mag + 1e-6)


@pytest.mark.parametrize("M,f,K", [(2048, 3328, 64), (1992, 3592, 96)])
def test_linear_dx_with_gated_activation_backward_in_the_epilogue(M, f, K):
    """dY . Wd (the gradient of the gated activation, never stored) turned into d gate | d up in the
    contraction's epilogue, against the oracle's swiglu_bwd on the float64 product."""
    import torch
    import paper_2401_15207_amd as H_
    from oracle import hift_oracle as O
    rng = np.random.default_rng(M + f + K + 1)
    dy = _bf16_round(rng.standard_normal((M, K)))
    wt = _bf16_round(rng.standard_normal((f, K)) / np.sqrt(K))           # rows = columns of the down projection
    pre = _bf16_round(rng.standard_normal((M, 2 * f)) * 1.5)
    dact = dy.astype(np.float64) @ wt.astype(np.float64).T
    dg_ref, du_ref = O.swiglu_bwd(dact, pre[:, :f].astype(np.float64), pre[:, f:].astype(np.float64))
    scratch = torch.empty(H_.kernel_packed_bytes(f, K) // 2, dtype=torch.bfloat16, device="cuda")
    out = torch.full((M, 2 * f), float("nan"), dtype=torch.bfloat16, device="cuda")
    H_.kernel_linear_fused(H_.EPILOGUE_SWIGLU_BWD, M, f, K, _dev(dy, True), K, _dev(wt, True), scratch, out, _dev(pre, True), None, 0, 0)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().astype(np.float64)
    ref = np.concatenate([dg_ref, du_ref], 1)
    # one bf16 rounding of the result; the fp32 accumulation of d act enters through its factor
    fac = np.abs(ref) / np.maximum(np.abs(np.concatenate([dact, dact], 1)), 1e-30)
    assert np.all(np.abs(got - ref) <= 2 ** -8 * np.abs(ref) + 1e-5 * fac * np.sqrt(K) + 1e-7)


@pytest.mark.parametrize("M,N,K,keep", [(2048, 3328, 256, 1), (1992, 3592, 96, 1), (2048, 20480, 64, 0)])
def test_linear_with_bias_and_gelu_in_the_epilogue(M, N, K, keep):
    """gelu(x . W^T + b) formed in the contraction's epilogue from the bf16-rounded pre-activations, against the
    oracle's erf-form GELU of those.  The kernel's erf has an absolute error below 1.5e-7, which gelu scales by |x| / 2."""
    import torch
    import paper_2401_15207_amd as H_
    from oracle import hift_oracle as O
    rng = np.random.default_rng(M + N + K + 2)
    x = _bf16_round(rng.standard_normal((M, K)))
    w = _bf16_round(rng.standard_normal((N, K)) * (2.0 / np.sqrt(K)))
    b = _bf16_round(rng.standard_normal(N))
    pre_ref = x.astype(np.float64) @ w.astype(np.float64).T + b
    scratch = torch.empty(H_.kernel_packed_bytes(N, K) // 2, dtype=torch.bfloat16, device="cuda")
    pre = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    act = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    H_.kernel_linear_gelu(0, M, N, K, _dev(x, True), K, _dev(w, True), _dev(b, True), scratch, pre if keep else None, act)
    torch.cuda.synchronize()
    a = act.float().cpu().numpy().astype(np.float64)
    if keep:
        p = pre.float().cpu().numpy().astype(np.float64)
        assert np.all(np.abs(p - pre_ref) <= 2 ** -8 * np.abs(pre_ref) + 1e-5)
        a_ref = O.gelu_fwd(p)
        assert np.all(np.abs(a - a_ref) <= 2 ** -8 * np.abs(a_ref) + 1e-6 * (1.0 + np.abs(p)))
    else:
        assert torch.isnan(pre.float()).all()
        p = _bf16_round(pre_ref).astype(np.float64)     # within one rounding of what the kernel held
        a_ref = O.gelu_fwd(p)
        slack = 2 ** -7 * (np.abs(a_ref) + np.abs(p) * 1.2)      # |gelu'| <= 1.13
        assert np.all(np.abs(a - a_ref) <= slack + 1e-6)


@pytest.mark.parametrize("M,N,K", [(2048, 3328, 64), (1992, 3592, 96)])
def test_linear_dx_with_gelu_backward_in_the_epilogue(M, N, K):
    """dY . W (the gradient of the activation, never stored) times gelu'(pre) in the contraction's epilogue, against
    the oracle's gelu_bwd on the float64 product."""
    import torch
    import paper_2401_15207_amd as H_
    from oracle import hift_oracle as O
    rng = np.random.default_rng(M + N + K + 4)
    dy = _bf16_round(rng.standard_normal((M, K)))
    wt = _bf16_round(rng.standard_normal((N, K)) / np.sqrt(K))           # rows = columns of the second projection
    pre = _bf16_round(rng.standard_normal((M, N)) * 2.0)
    dact = dy.astype(np.float64) @ wt.astype(np.float64).T
    ref = O.gelu_bwd(dact, pre.astype(np.float64))
    scratch = torch.empty(H_.kernel_packed_bytes(N, K) // 2, dtype=torch.bfloat16, device="cuda")
    out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    H_.kernel_linear_gelu(1, M, N, K, _dev(dy, True), K, _dev(wt, True), None, scratch, out, _dev(pre, True))
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().astype(np.float64)
    # one bf16 rounding; the fp32 accumulation of d act and the 1e-6 of the derivative enter through |d act|
    assert np.all(np.abs(got - ref) <= 2 ** -8 * np.abs(ref) + 1e-5 * np.sqrt(K) * 1.2 + 2e-6 * np.abs(dact) + 1e-7)


@pytest.mark.parametrize("M,N,K", [(2048, 5120, 2048), (2048, 5632, 1024), (1990, 4392, 1024)])
def test_gemm_with_packed_weight_operand_and_shared_last_round(M, N, K):
    """Tiles of the last, partial round shared by 2 to 4 workgroups along K and summed by the last one to
    finish: against the float64 product, twice in a row on the same work space (the counters must come
    back to zero), and bit-identical between the two calls (the sum is taken in a fixed order)."""
    import torch
    import paper_2401_15207_amd as H
    rng = np.random.default_rng(M + N + K)
    A = _bf16_round(rng.standard_normal((M, K)))
    B = _bf16_round(rng.standard_normal((N, K)) * 0.5)
    bias = _bf16_round(rng.standard_normal(N))
    R = _bf16_round(rng.standard_normal((M, N)))
    ref = A.astype(np.float64) @ B.astype(np.float64).T + bias + R
    dBp = torch.empty(H.kernel_packed_bytes(N, K) // 2, dtype=torch.bfloat16, device="cuda")
    H.kernel_pack_b(1, N, K, _dev(B, True), K, dBp)
    ws = torch.zeros(H.kernel_packed_workspace_bytes() // 4, dtype=torch.float32, device="cuda")
    ws[256:] = float("nan")                     # only the counters need to start at zero
    dA = _dev(A, True)
    for out_f32 in (0, 1):
        outs = []
        for _rep in range(2):
            dC = torch.zeros((M, N), dtype=torch.float32 if out_f32 else torch.bfloat16, device="cuda")
            H.kernel_gemm_packed_ws(out_f32, M, N, K, dA, K, dBp, dC, N, _dev(bias, True), _dev(R, not out_f32), ws)
            torch.cuda.synchronize()
            assert int(ws[:256].view(torch.int32).abs().sum()) == 0
            outs.append(dC.float().cpu().numpy())
        assert np.array_equal(outs[0], outs[1])
        got = outs[0].astype(np.float64)
        scale = np.sqrt(K) + 1.0
        tol = (1e-5 if out_f32 else 2 ** -8) * (np.abs(ref) + (scale if out_f32 else 0.02 * scale))
        bad = np.abs(got - ref) > tol
        assert not bad.any(), (out_f32, int(bad.sum()), float(np.max(np.abs(got - ref))))


@pytest.mark.parametrize("M,N,K,shared", [(2048, 3328, 256, 0), (1990, 3328, 96, 0), (2048, 5120, 1024, 1)])
def test_packed_gemm_leaves_row_sums_of_squares(M, N, K, shared):
    """The contraction that writes rows x = A . B^T + R (bf16) also leaves, per row and 64-column strip, the sum of
    squares of the values it stored: against the float64 product.  A stored value is within one bf16 rounding
    (2^-9 relative, plus the accumulation) of the exact one, its square within 2^-8."""
    import torch
    import paper_2401_15207_amd as H
    rng = np.random.default_rng(M + N + K + 5)
    A = _bf16_round(rng.standard_normal((M, K)))
    B = _bf16_round(rng.standard_normal((N, K)) * 0.5)
    R = _bf16_round(rng.standard_normal((M, N)) * 3.0)
    ref = A.astype(np.float64) @ B.astype(np.float64).T + R
    dBp = torch.empty(H.kernel_packed_bytes(N, K) // 2, dtype=torch.bfloat16, device="cuda")
    H.kernel_pack_b(1, N, K, _dev(B, True), K, dBp)
    ws = torch.zeros(H.kernel_packed_workspace_bytes() // 4, dtype=torch.float32, device="cuda") if shared else None
    dC = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    sq = torch.full((M, N // 64), float("nan"), dtype=torch.float32, device="cuda")
    H.kernel_gemm_packed_rowsq(M, N, K, _dev(A, True), K, dBp, dC, N, _dev(R, True), sq, ws)
    torch.cuda.synchronize()
    got = dC.float().cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ref) <= 2 ** -8 * np.abs(ref) + 1e-5 * np.sqrt(K))
    q = sq.cpu().numpy().astype(np.float64)
    q_ref = (ref ** 2).reshape(M, N // 64, 64).sum(-1)
    assert np.all(np.abs(q - q_ref) <= 2 ** -7 * q_ref + 1e-4)
    # and exactly (up to the order of the fp32 sum) the squares of what was stored
    q_own = (got ** 2).reshape(M, N // 64, 64).sum(-1)
    assert np.all(np.abs(q - q_own) <= 1e-5 * q_own + 1e-12)


@pytest.mark.parametrize("rows,d,n", [(2048, 4096, 64), (77, 5120, 80), (3, 520, 9), (0, 64, 1)])
def test_row_sums_of_squares(rows, d, n):
    import torch
    import paper_2401_15207_amd as H
    rng = np.random.default_rng(rows + d)
    x = _bf16_round(rng.standard_normal((rows, d)) * 2.0)
    out = torch.full((rows, n), float("nan"), dtype=torch.float32, device="cuda")
    H.kernel_row_sumsq(rows, d, _dev(x, True), n, out)
    torch.cuda.synchronize()
    o = out.cpu().numpy().astype(np.float64)
    ref = (x.astype(np.float64) ** 2).sum(-1)
    assert np.all(np.abs(o[:, 0] - ref) <= 1e-5 * ref)
    assert np.all(o[:, 1:] == 0.0)


def _norm_fold_slack(x, rstd, g, w):
    """Bound on what rounding gain * W to bf16 can move rstd x . (gain W)^T: 2^-9 of the sum of magnitudes."""
    return 2 ** -9 * ((np.abs(x) * rstd) @ np.abs(g[None, :] * w).T)


@pytest.mark.parametrize("M,f,K,shared", [(2048, 1664, 512, 0), (1992, 1792, 1024, 0), (2048, 2560, 1024, 1)])
def test_linear_with_rms_normalisation_folded_and_gated_activation(M, f, K, shared):
    """silu(gate) * up of rmsnorm(x, gain) . [Wg | Wu]^T, computed from x, gain * W and the row sums of squares,
    against the oracle's rmsnorm and swiglu on the float64 product."""
    import torch
    import paper_2401_15207_amd as H_
    from oracle import hift_oracle as O
    rng = np.random.default_rng(M + f + K + 9)
    x = _bf16_round(rng.standard_normal((M, K)) * rng.uniform(0.3, 6.0, (M, 1)))
    g = _bf16_round(1.0 + 0.3 * rng.standard_normal(K))
    w = _bf16_round(rng.standard_normal((2 * f, K)) * (1.5 / np.sqrt(K)))
    eps = 1e-5
    h, (_, rstd) = O.rmsnorm_fwd(x.astype(np.float64), g.astype(np.float64), eps)
    pre_ref = h @ w.astype(np.float64).T
    slack = _norm_fold_slack(x.astype(np.float64), rstd, g.astype(np.float64), w.astype(np.float64))
    dx = _dev(x, True)
    sq = torch.empty((M, K // 64), dtype=torch.float32, device="cuda")
    H_.kernel_row_sumsq(M, K, dx, K // 64, sq)
    scratch = torch.empty(H_.kernel_packed_bytes(2 * f, K) // 2, dtype=torch.bfloat16, device="cuda")
    pre = torch.full((M, 2 * f), float("nan"), dtype=torch.bfloat16, device="cuda")
    act = torch.full((M, f), float("nan"), dtype=torch.bfloat16, device="cuda")
    stats = torch.full((M, 2), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.zeros(H_.kernel_packed_workspace_bytes() // 4, dtype=torch.float32, device="cuda") if shared else None
    H_.kernel_linear_norm_fused(H_.EPILOGUE_SWIGLU, M, 2 * f, K, dx, K, _dev(w, True), _dev(g, True), scratch, pre, act,
                                None, 0, 0, sq, eps, stats, ws)
    torch.cuda.synchronize()
    st = stats.cpu().numpy().astype(np.float64)
    assert np.all(st[:, 0] == 0.0)
    assert np.all(np.abs(st[:, 1] - rstd[:, 0]) <= 1e-5 * rstd[:, 0])
    p = pre.float().cpu().numpy().astype(np.float64)
    assert np.all(np.abs(p - pre_ref) <= 2 ** -8 * np.abs(pre_ref) + slack + 1e-5)
    a = act.float().cpu().numpy().astype(np.float64)
    a_ref = O.swiglu_fwd(p[:, :f], p[:, f:])          # the activation is formed from the stored pre-activations
    assert np.all(np.abs(a - a_ref) <= 2 ** -8 * np.abs(a_ref) + 1e-6)


@pytest.mark.parametrize("M,S,heads,K", [(2048, 512, 10, 512), (1000, 200, 18, 1024)])
def test_linear_with_rms_normalisation_folded_and_rotary_embedding(M, S, heads, K):
    """rope(rmsnorm(x, gain) . Wqkv^T) from x, gain * W and the row sums of squares, against the oracle's
    rmsnorm and rope on the float64 product."""
    import torch
    import paper_2401_15207_amd as H_
    from oracle import hift_oracle as O
    hd, d = 128, heads * 128
    N = 3 * d
    rng = np.random.default_rng(M + S + heads + K + 3)
    x = _bf16_round(rng.standard_normal((M, K)) * rng.uniform(0.3, 6.0, (M, 1)))
    g = _bf16_round(1.0 + 0.3 * rng.standard_normal(K))
    w = _bf16_round(rng.standard_normal((N, K)) / np.sqrt(K))
    eps = 1e-6
    h, (_, rstd) = O.rmsnorm_fwd(x.astype(np.float64), g.astype(np.float64), eps)
    y_ref = h @ w.astype(np.float64).T
    slack = _norm_fold_slack(x.astype(np.float64), rstd, g.astype(np.float64), w.astype(np.float64))
    cos, sin = O.rope_angles(S, hd, 10000.0, np.float64)
    pos = np.arange(M) % S
    rot_cols = 2 * d

    def heads_of(a):
        return a[:, :rot_cols].reshape(M, 2 * heads, hd).transpose(1, 0, 2)

    blk = heads_of(y_ref)
    mag = np.abs(y_ref).copy()
    mag[:, :rot_cols] = (np.abs(blk) + np.abs(np.roll(blk, hd // 2, axis=-1))).transpose(1, 0, 2).reshape(M, rot_cols)
    sblk = heads_of(slack)
    slack[:, :rot_cols] = (sblk + np.roll(sblk, hd // 2, axis=-1)).transpose(1, 0, 2).reshape(M, rot_cols)
    y_ref[:, :rot_cols] = O.rope_fwd(blk, cos[pos], sin[pos]).transpose(1, 0, 2).reshape(M, rot_cols)
    tab = torch.from_numpy(np.stack([cos, sin], -1).astype(np.float32)).cuda().contiguous()
    dx = _dev(x, True)
    sq = torch.empty((M, K // 64), dtype=torch.float32, device="cuda")
    H_.kernel_row_sumsq(M, K, dx, K // 64, sq)
    scratch = torch.empty(H_.kernel_packed_bytes(N, K) // 2, dtype=torch.bfloat16, device="cuda")
    y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    stats = torch.full((M, 2), float("nan"), dtype=torch.float32, device="cuda")
    H_.kernel_linear_norm_fused(H_.EPILOGUE_ROPE, M, N, K, dx, K, _dev(w, True), _dev(g, True), scratch, y, None, tab, S,
                                rot_cols, sq, eps, stats)
    torch.cuda.synchronize()
    st = stats.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(st[:, 1] - rstd[:, 0]) <= 1e-5 * rstd[:, 0])
    got = y.float().cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - y_ref) <= 2 ** -8 * np.abs(y_ref) + slack + 1e-5 * mag + 1e-6)


@pytest.mark.parametrize("B,H,S,hd,causal,rope", [(2, 3, 200, 64, 1, 1), (1, 2, 512, 128, 1, 1), (2, 2, 136, 128, 0, 0),
                                                   (1, 2, 72, 64, 1, 0), (1, 1, 8, 128, 1, 1), (2, 4, 384, 64, 0, 1),
                                                   (4, 32, 512, 128, 1, 1)])
def test_fused_attention_backward(B, H, S, hd, causal, rope):
    """Query-major and key-major kernels against the oracle's attention backward, followed (rope) by the oracle's
    adjoint of the rotary embedding on dq and dk.  The kernels get what the forward leaves: the context (bf16) and
    log2 of each row's sum of exponentials, both computed here on the CPU; they form the probabilities again from
    q, k and the log-sums.  The row sum D_i = sum_j dP.P is taken as dO_i.O_i with the context as stored (bf16:
    each entry off by up to 2^-9 of itself), so D_i is off by up to delta_i = 2^-9 sum_e |dO_ie O_ie|, dS_ij by
    scale delta_i P_ij, and dQ, dK by the sums of that through K and Q; the tolerance allows twice this.  P and dS
    enter their products rounded to bf16 (2^-9 relative per entry): dV, dQ, dK may be off by 2^-9 times the sums
    of |P| |dO|, |dS| |K|, |dS| |Q|; then one rounding of the outputs."""
    import torch
    from scipy.special import logsumexp
    import paper_2401_15207_amd as H_
    from oracle import hift_oracle as O
    rng = np.random.default_rng(11 + B * 1000 + S + hd + causal)
    d = H * hd
    full = B * H * S * S <= 2 ** 22     # the oracle in float64 on everything; else on two (batch, head) pairs
    qkv = _bf16_round(rng.standard_normal((B * S, 3 * d)) * (1.5 if full else 1.0))
    dctx = _bf16_round(rng.standard_normal((B * S, d)))
    heads = lambda a: a.reshape(B, S, H, hd).transpose(0, 2, 1, 3).astype(np.float64)
    q, k, v, do = heads(qkv[:, :d]), heads(qkv[:, d:2 * d]), heads(qkv[:, 2 * d:]), heads(dctx)
    ctx_ref, p = O.attention_fwd(q, k, v, bool(causal))
    ctx = _bf16_round(ctx_ref)
    ctx_rows = np.ascontiguousarray(ctx.transpose(0, 2, 1, 3).reshape(B * S, d))
    sc = np.matmul(q, np.swapaxes(k, -1, -2)) / np.sqrt(hd)
    if causal:
        sc = np.where(np.tril(np.ones((S, S), bool)), sc, -np.inf)
    lse = (logsumexp(sc, axis=-1) / np.log(2.0)).astype(np.float32)
    cos, sin = O.rope_angles(S, hd, 10000.0, np.float64)
    tab = torch.from_numpy(np.stack([cos, sin], -1).astype(np.float32)).cuda().contiguous() if rope else None
    d_sum = torch.full((B * H * S,), float("nan"), dtype=torch.float32, device="cuda")
    d_dqkv = torch.full((B * S, 3 * d), float("nan"), dtype=torch.bfloat16, device="cuda")
    H_.kernel_attention_bwd(B, H, S, hd, causal, _dev(qkv, True), _dev(ctx_rows, True),
                            torch.from_numpy(np.ascontiguousarray(lse.reshape(-1))).cuda(), _dev(dctx, True), d_sum, d_dqkv, tab)
    torch.cuda.synchronize()
    out = d_dqkv.float().cpu().numpy()
    assert np.isfinite(out).all()
    dsum_ref = (do * ctx.astype(np.float64)).sum(-1)
    assert np.all(np.abs(d_sum.cpu().numpy().reshape(B, H, S) - dsum_ref) <= 1e-5 * np.abs(do * ctx).sum(-1) + 1e-6)
    dq, dk, dv = heads(out[:, :d]), heads(out[:, d:2 * d]), heads(out[:, 2 * d:])
    pairs = [(b, h) for b in range(B) for h in range(H)] if full else [(0, 0), (B - 1, H - 1)]
    for b, h in pairs:
        dq_ref, dk_ref, dv_ref = O.attention_bwd(do[b, h], q[b, h], k[b, h], v[b, h], p[b, h])
        delta = 2.0 ** -8 * np.abs(do[b, h] * ctx[b, h]).sum(-1, keepdims=True) / np.sqrt(hd)
        dp = do[b, h] @ v[b, h].T
        ds_abs = np.abs(p[b, h] * (dp - (dp * p[b, h]).sum(-1, keepdims=True))) / np.sqrt(hd)
        slack_q = delta * np.abs(p[b, h] @ k[b, h]) + 2.0 ** -9 * (ds_abs @ np.abs(k[b, h]))
        slack_k = (p[b, h] * delta).T @ np.abs(q[b, h]) + 2.0 ** -9 * (ds_abs.T @ np.abs(q[b, h]))
        slack_v = 2.0 ** -9 * (p[b, h].T @ np.abs(do[b, h]))
        if rope:
            dq_ref, dk_ref = O.rope_bwd(dq_ref, cos, sin), O.rope_bwd(dk_ref, cos, sin)
            mix = lambda s: s + np.roll(s, hd // 2, axis=-1)       # a rotated entry mixes the two of its pair
            slack_q, slack_k = mix(slack_q), mix(slack_k)
        for name, got, ref, slack in (("dq", dq[b, h], dq_ref, slack_q), ("dk", dk[b, h], dk_ref, slack_k),
                                      ("dv", dv[b, h], dv_ref, slack_v)):
            rms = np.sqrt(np.mean(ref ** 2))
            err = np.abs(got - ref)
            bad = err > 2 ** -7 * np.abs(ref) + 2e-2 * rms + slack + 1e-6
            assert not bad.any(), (name, b, h, int(bad.sum()), float(err.max()), float(rms))
            assert np.sqrt(np.mean(err ** 2)) <= 5e-3 * rms + np.sqrt(np.mean(np.square(slack))) + 1e-6, (name, b, h)
