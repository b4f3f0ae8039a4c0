"""GPU test of the allocation-free entry point oz2_dgemm_noalloc: through the C ABI, against
oz2_dgemm on the same inputs, two calls in a row (the second smaller, in the same fixed
workspace), and the refusal of sizes beyond the fixed workspace."""
import numpy as np
import pytest

import synth_inputs as S

pytestmark = pytest.mark.gpu

TOL64 = 1e-14


def test_noalloc_entry_point_equals_oz2_dgemm():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    import paper_2508_03984_amd as oz
    from paper_2508_03984_amd import binding as b
    oz.load()
    cases = [(1000, 900, 1000, 16, 0.5, 1.0, 0.0),          # close to the limit of the fixed workspace
             (300, 200, 333, 14, 1.0, -0.5, 2.0)]           # smaller, right after it, with alpha and beta
    prepared = []
    for m, n, k, N, phi, alpha, beta in cases:
        assert oz.oz2_workspace_bytes(m, n, k, N) <= b.OZ2_NOALLOC_WORKSPACE_BYTES
        A, B = S.gemm_inputs(m, n, k, phi, seed=300 + m)
        Cin = S.matrix(m, n, 0.5, seed=301 + m)
        dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
        want = torch.from_numpy(Cin).cuda()
        oz.oz2_dgemm(m, n, k, alpha, dA, k, dB, n, beta, want, n, N)
        got = torch.from_numpy(Cin).cuda()
        prepared.append((m, n, k, N, alpha, beta, dA, dB, want, got))
    # The first call on a device looks the fixed array up; the runtime materialises the array on
    # that occasion (it belongs to the library's device image).  From then on nothing may change.
    m, n, k, N, alpha, beta, dA, dB, want, got = prepared[1]
    warm = got.clone()
    oz.oz2_dgemm_noalloc(m, n, k, alpha, dA, k, dB, n, beta, warm, n, N)
    torch.cuda.synchronize()
    assert torch.equal(warm, want)
    free_before = torch.cuda.mem_get_info()[0]
    for m, n, k, N, alpha, beta, dA, dB, want, got in prepared:      # back to back, no synchronisation between
        oz.oz2_dgemm_noalloc(m, n, k, alpha, dA, k, dB, n, beta, got, n, N)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before                # nothing was allocated on the device
    for m, n, k, N, alpha, beta, dA, dB, want, got in prepared:
        w, g = want.cpu().numpy(), got.cpu().numpy()
        rel = np.max(np.abs(g - w) / np.where(w == 0, 1.0, np.abs(w)))
        assert rel <= TOL64, (m, n, k, rel)
        assert np.array_equal(g, w)                                   # same kernels, same order: identical
    # beyond the fixed workspace: refused with a status, C untouched
    m = n = k = 2048
    assert oz.oz2_workspace_bytes(m, n, k, 16) > b.OZ2_NOALLOC_WORKSPACE_BYTES
    dA = torch.ones((m, k), dtype=torch.float64, device="cuda")
    dC = torch.full((m, n), 7.0, dtype=torch.float64, device="cuda")
    with pytest.raises(oz.OZ2Error) as e:
        oz.oz2_dgemm_noalloc(m, n, k, 1.0, dA, k, dA, n, 0.0, dC, n, 16)
    assert e.value.status == 3
    torch.cuda.synchronize()
    assert bool((dC == 7.0).all())
    # empty products and k = 0 behave as in oz2_dgemm
    oz.oz2_dgemm_noalloc(0, n, k, 1.0, dA, k, dA, n, 0.0, dC, n, 16)
    oz.oz2_dgemm_noalloc(4, 4, 0, 1.0, dA, 1, dA, 4, 0.5, dC, n, 16)
    torch.cuda.synchronize()
    assert bool((dC[:4, :4] == 3.5).all()) and float(dC[4, 4]) == 7.0
    oz.oz2_release()
