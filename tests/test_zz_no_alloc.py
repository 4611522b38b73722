"""bita_gemm_noalloc (GPU): the entry point for callers that cannot allocate.  Its kernels are
those of bita_gemm, its scratch a static device array: the result must equal bita_gemm's bit for
bit, also on a second, smaller call that finds the first call's data in the scratch."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _case(bita, B, M, N, K, seed, two_planes):
    g = torch.Generator().manual_seed(seed)
    a32 = torch.randn(M, K, generator=g)
    hi = a32.to(torch.bfloat16)
    lo = (a32 - hi.float()).to(torch.bfloat16) if two_planes else None
    w = (torch.randn(N, K, generator=g) * 0.05).to(torch.bfloat16)
    wp = bita.pack_weight(w.cuda())
    hi_d, lo_d = hi.cuda(), (lo.cuda() if two_planes else None)
    ref = bita.gemm(hi_d, wp, N, a_lo=lo_d)                  # the existing entry point, workspace from torch
    out = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    B.gemm_noalloc(hi_d, wp, N, out, a_lo=lo_d)
    torch.cuda.synchronize()
    assert torch.equal(out, ref), (M, N, K)
    # and both match the float64 product of the operands as given
    a64 = hi.to(torch.float64) + (lo.to(torch.float64) if two_planes else 0.0)
    exact = a64.numpy() @ w.to(torch.float64).numpy().T
    assert np.abs(out.cpu().numpy() - exact).max() <= 2e-5 * np.abs(exact).max() + 1e-6


def test_noalloc_gemm_equals_gemm_on_two_calls_in_a_row():
    import paper_2401_12522_amd as bita
    from paper_2401_12522_amd import binding as B
    L = bita.lib()
    assert L.bita_gemm_noalloc_max_scratch_bytes() == 32 << 20
    # first call: split-K partials and a five-tile slab fill a good part of the scratch
    assert 4 << 20 < L.bita_gemm_noalloc_scratch_bytes(68, 4096, 4096) <= 32 << 20
    _case(bita, B, 68, 4096, 4096, 1, True)
    # second call, smaller in every dimension, a different plan (other split count, one m-tile,
    # packed last tile): whatever the first call left in the scratch must not matter
    _case(bita, B, 5, 1024, 1376, 2, True)
    # a single-plane call and a single-split one after those
    _case(bita, B, 12, 256, 688, 3, False)
    _case(bita, B, 68, 22016, 512, 4, True)


def test_noalloc_gemm_rejects_what_the_static_scratch_cannot_hold():
    import paper_2401_12522_amd as bita
    from paper_2401_12522_amd import binding as B
    L = bita.lib()
    M, N, K = 512, 1024, 28672
    assert L.bita_gemm_noalloc_scratch_bytes(M, N, K) > L.bita_gemm_noalloc_max_scratch_bytes()
    a = torch.zeros((M, K), dtype=torch.bfloat16, device="cuda")
    wp = torch.zeros(bita.packed_bytes(N, K), dtype=torch.uint8, device="cuda")
    out = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    with pytest.raises(B.BitaError) as e:
        B.gemm_noalloc(a, wp, N, out)
    assert e.value.code == -3 and "scratch" in str(e.value)
