"""The contraction with a shared last round through the entry point that allocates nothing
(hift_kernel_gemm_packed_static: work space built into the library) against the entry point that takes the
caller's work space, through the C ABI: two calls in a row, the second on a smaller problem."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _bf16(x):
    from hift_inputs import round_to_bf16
    return round_to_bf16(x.astype(np.float32))


def test_static_work_space_matches_caller_work_space_two_calls_second_smaller():
    import torch
    import paper_2401_15207_amd as H
    ws = torch.zeros(H.kernel_packed_workspace_bytes() // 4, dtype=torch.float32, device="cuda")
    # (2048, 5120, 2048): 320 tiles, the last 64 shared four ways; (1990, 4392, 1024): ragged edges, 288 tiles,
    # the last 32 shared four ways; (2048, 4096, 512): whole rounds only, no work space used at all
    for M, N, K in [(2048, 5120, 2048), (1990, 4392, 1024), (2048, 4096, 512)]:
        rng = np.random.default_rng(M + N + K)
        A = _bf16(rng.standard_normal((M, K)))
        B = _bf16(rng.standard_normal((N, K)) * 0.5)
        bias = _bf16(rng.standard_normal(N))
        R = _bf16(rng.standard_normal((M, N)))
        ref = A.astype(np.float64) @ B.astype(np.float64).T + bias + R
        dA = torch.from_numpy(A).cuda().to(torch.bfloat16)
        dB = torch.from_numpy(B).cuda().to(torch.bfloat16)
        dbias = torch.from_numpy(bias).cuda().to(torch.bfloat16)
        dBp = torch.empty(H.kernel_packed_bytes(N, K) // 2, dtype=torch.bfloat16, device="cuda")
        H.kernel_pack_b(1, N, K, dB, K, dBp)
        for out_f32 in (0, 1):
            dR = torch.from_numpy(R).cuda()
            if not out_f32:
                dR = dR.to(torch.bfloat16)
            want = torch.zeros((M, N), dtype=torch.float32 if out_f32 else torch.bfloat16, device="cuda")
            got = torch.full_like(want, float("nan"))
            H.kernel_gemm_packed_ws(out_f32, M, N, K, dA, K, dBp, want, N, dbias, dR, ws)
            H.kernel_gemm_packed_static(out_f32, M, N, K, dA, K, dBp, got, N, dbias, dR)
            torch.cuda.synchronize()
            # the partial tiles are summed in a fixed order: the two entry points agree bit for bit
            assert torch.equal(got, want), (M, N, K, out_f32)
            g = got.float().cpu().numpy().astype(np.float64)
            scale = np.sqrt(K) + 1.0
            tol = (1e-5 if out_f32 else 2 ** -8) * (np.abs(ref) + (scale if out_f32 else 0.02 * scale))
            assert not (np.abs(g - ref) > tol).any(), (M, N, K, out_f32, float(np.max(np.abs(g - ref))))


def test_static_work_space_rejects_what_the_kernel_does_not_take():
    import torch
    import paper_2401_15207_amd as H
    x = torch.zeros(64 * 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(H.HiftError):
        H.kernel_gemm_packed_static(0, 64, 64, 64, x, 64, x, x, 64)     # far too few tiles for this kernel
