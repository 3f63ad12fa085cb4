"""The entry point that allocates nothing (vf_gemm_noalloc) against vf_gemm: the same sliced
contraction, the slabs added in slab order, bit for bit; two calls in a row, the second with a
smaller input, all calls sharing the library's static device scratch."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _operands(M, N, K, seed):
    import torch
    rng = np.random.Generator(np.random.PCG64(seed))
    A = torch.from_numpy(rng.standard_normal((M, K)).astype(np.float32)).to(torch.bfloat16).cuda()
    B = torch.from_numpy(rng.standard_normal((N, K)).astype(np.float32)).to(torch.bfloat16).cuda()
    return A, B


def _via_vf_gemm(A, B, M, N, K, alpha, nsplit, c0=None):
    """vf_gemm's slabs added in slab order on the host in fp32, then the one fused multiply-add."""
    import torch
    import paper_2009_09523_amd as vf
    slabs = torch.full((nsplit, M, N), 9.0, device="cuda")
    vf.vf_gemm(A, B, slabs, M, N, K, nsplit=nsplit)
    torch.cuda.synchronize()
    s = slabs.cpu().numpy()
    v = s[0].copy()
    for k in range(1, nsplit):
        v = (v + s[k]).astype(np.float32)
    old = np.zeros((M, N)) if c0 is None else c0.astype(np.float64)
    return (np.float64(np.float32(alpha)) * v.astype(np.float64) + old).astype(np.float32)   # fma: one rounding


def test_noalloc_matches_vf_gemm_on_two_calls_in_a_row():
    import torch
    import paper_2009_09523_amd as vf
    # first call: node-sized product in 16 slices, the whole scratch (16 x 128 x 4096 floats = 32 MiB)
    M, N, K, nsplit = 128, 4096, 4096, 16
    assert nsplit * M * N * 4 == vf.VF_NOALLOC_SCRATCH_BYTES
    A, B = _operands(M, N, K, 1)
    C1 = torch.full((M, N), 3.0, device="cuda")
    assert vf.vf_gemm_noalloc(A, B, C1, M, N, K, alpha=0.5, nsplit=nsplit) == 0
    # second call right behind it on the same stream: smaller and ragged, accumulating
    m, n, k, ns = 48, 1000, 520, 3
    a, b = _operands(m, n, k, 2)
    rng = np.random.Generator(np.random.PCG64(3))
    c0 = rng.standard_normal((m, n)).astype(np.float32)
    C2 = torch.from_numpy(c0).cuda()
    assert vf.vf_gemm_noalloc(a, b, C2, m, n, k, alpha=-1.25, accumulate=True, nsplit=ns) == 0
    torch.cuda.synchronize()
    got1, got2 = C1.cpu().numpy(), C2.cpu().numpy()
    want1 = _via_vf_gemm(A, B, M, N, K, 0.5, nsplit)
    want2 = _via_vf_gemm(a, b, m, n, k, -1.25, ns, c0)
    np.testing.assert_array_equal(got1, want1)
    np.testing.assert_array_equal(got2, want2)
    # and against the plain definition
    ref = A.double().cpu().numpy() @ B.double().cpu().numpy().T
    assert np.max(np.abs(got1 - 0.5 * ref)) <= 1e-5 * np.sqrt(K) * np.max(np.abs(ref))
    # a third call, one slice: the scratch holds the whole product once
    C3 = torch.empty((m, n), device="cuda")
    assert vf.vf_gemm_noalloc(a, b, C3, m, n, k, nsplit=1) == 0
    torch.cuda.synchronize()
    np.testing.assert_array_equal(C3.cpu().numpy(), _via_vf_gemm(a, b, m, n, k, 1.0, 1))


def test_noalloc_rejects_what_does_not_fit():
    import torch
    import paper_2009_09523_amd as vf
    from paper_2009_09523_amd.binding import VF_EINVAL
    M, N, K = 128, 4096, 4096
    A, B = _operands(M, N, K, 4)
    C = torch.full((M, N), 7.0, device="cuda")
    assert vf.vf_gemm_noalloc(A, B, C, M, N, K, nsplit=17) == VF_EINVAL      # 17 slabs: beyond the scratch
    assert vf.vf_gemm_noalloc(A, B, C, M, N, K, nsplit=0) == VF_EINVAL
    torch.cuda.synchronize()
    assert torch.all(C == 7.0)                                              # nothing was enqueued
