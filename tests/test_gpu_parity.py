"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the
same seeded inputs.  Integer stages (shifts, residues, INT32 products) must be
bit-exact; the final C must agree to 1e-14 relative (FP64 path) or 2^-23 (FP32
path) -- both sides start from identical integers and run the same IEEE
operations, so the expected difference is zero."""
import os

import numpy as np
import pytest

import synth_inputs as S

pytestmark = pytest.mark.gpu

TOL64 = 1e-14
TOL32 = 2.0 ** -23


@pytest.fixture(scope="module")
def oz():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2508_03984_amd as oz
    oz.load()                      # raises if liboz2.so has not been built: no fallback
    yield oz
    oz.oz2_release()


def gpu_gemm(oz, A, B, N, alpha=1.0, beta=0.0, Cin=None, lda=None, ldb=None, accurate=False,
             int32_products=False, ldc=None, c_offset=0, small_conversion=True):
    """Run oz2_dgemm / oz2_sgemm and fetch every stage, trimmed to the logical shapes.  By
    default the GEMM emits U_s (uint8); with int32_products the diagnostic form C'_s.
    small_conversion=False: the general conversion kernels also at these small sizes."""
    import torch
    m, k = A.shape
    n = B.shape[1]
    dt = torch.float64 if A.dtype == np.float64 else torch.float32
    lda = lda or k
    ldb = ldb or n
    dA = torch.zeros((m, lda), dtype=dt, device="cuda"); dA[:, :k] = torch.from_numpy(A).cuda()
    dB = torch.zeros((k, ldb), dtype=dt, device="cuda"); dB[:, :n] = torch.from_numpy(B).cuda()
    ldc = ldc or n
    store = torch.full((m * ldc + c_offset,), float("nan"), dtype=dt, device="cuda")
    dC = store[c_offset:].view(m, ldc)[:, :n]               # row stride ldc, start offset c_offset
    if Cin is not None:
        dC.copy_(torch.from_numpy(np.ascontiguousarray(Cin)).cuda())
    if accurate:
        fn = oz.oz2_dgemm_accurate if dt == torch.float64 else oz.oz2_sgemm_accurate
    else:
        fn = oz.oz2_dgemm if dt == torch.float64 else oz.oz2_sgemm
    oz.oz2_set_int32_products(int32_products)
    oz.oz2_set_small_conversion(small_conversion)
    try:
        fn(m, n, k, alpha, dA, lda, dB, ldb, beta, dC, ldc, N)
    finally:
        oz.oz2_set_int32_products(False)
        oz.oz2_set_small_conversion(True)
    torch.cuda.synchronize()
    from paper_2508_03984_amd import binding as b
    out = dict(C=dC.cpu().numpy())
    if ldc > n:                                              # the gap between rows is untouched
        assert bool(torch.isnan(store[c_offset:].view(m, ldc)[:, n:]).all())
    out["tA"] = oz.stage_tensor(b.OZ2_STAGE_SHIFT_A).cpu().numpy()
    out["tB"] = oz.stage_tensor(b.OZ2_STAGE_SHIFT_B).cpu().numpy()
    ra = oz.unblock_slices(oz.stage_tensor(b.OZ2_STAGE_RES_A))
    rb = oz.unblock_slices(oz.stage_tensor(b.OZ2_STAGE_RES_B))
    if int32_products:
        out["prod"] = oz.stage_tensor(b.OZ2_STAGE_PROD)[:, :m, :n].cpu().numpy()
        with pytest.raises(oz.OZ2Error):
            oz.oz2_stage_ptr(b.OZ2_STAGE_U)
    else:
        out["U"] = oz.stage_tensor(b.OZ2_STAGE_U)[:, :m, :n].cpu().numpy()
        with pytest.raises(oz.OZ2Error):
            oz.oz2_stage_ptr(b.OZ2_STAGE_PROD)
    out["pad_clean"] = bool((ra[:, m:, :] == 0).all() and (ra[:, :, k:] == 0).all()
                            and (rb[:, n:, :] == 0).all() and (rb[:, :, k:] == 0).all())
    out["Ares"] = ra[:, :m, :k].cpu().numpy()
    out["Bres"] = rb[:, :n, :k].cpu().numpy()
    return out


def assert_parity(got, ref, is_double):
    assert np.array_equal(got["tA"], ref["tA"]), "row shifts differ"
    assert np.array_equal(got["tB"], ref["tB"]), "column shifts differ"
    assert got["pad_clean"], "padding of the residue slices is not zero"
    assert np.array_equal(got["Ares"], ref["Ares"]), "residues of A differ"
    assert np.array_equal(got["Bres"], ref["Bres"]), "residues of B differ"
    if "prod" in got:
        assert np.array_equal(got["prod"], ref["prod"]), "INT32 products differ"
    if "U" in got:
        assert np.array_equal(got["U"], ref["U"]), "reduced products U_s differ"
    c, r = got["C"].astype(np.float64), ref["C"].astype(np.float64)
    denom = np.where(r == 0, 1.0, np.abs(r))
    rel = np.max(np.abs(c - r) / denom) if c.size else 0.0
    assert rel <= (TOL64 if is_double else TOL32), f"C differs: max rel {rel}"
    assert np.array_equal(c == 0, r == 0)


CASES = [
    # m, n, k, N, phi, dtype
    (256, 256, 256, 14, 0.5, np.float64),      # the small configuration of the benchmark set
    (1, 1, 1, 2, 0.5, np.float64),
    (3, 5, 7, 20, 0.5, np.float64),
    (300, 200, 333, 16, 0.5, np.float64),      # ragged in every dimension
    (520, 390, 1000, 12, 2.0, np.float64),     # several tiles, one reduction round
    (257, 513, 129, 13, 1.0, np.float64),      # first N with two reduction rounds
    (130, 260, 640, 20, 4.0, np.float64),      # widest integers
    (256, 256, 256, 8, 0.5, np.float32),
    (300, 200, 333, 5, 1.0, np.float32),
    (97, 515, 1030, 9, 0.5, np.float32),
    (64, 64, 512, 2, 0.5, np.float32),
    (70, 66, 300, 20, 0.5, np.float32),        # more moduli than FP32 needs: still exact
    # rows of A long enough for every form of the shift kernel that reads a row once
    (40, 50, 2000, 14, 0.5, np.float64),       # 128 threads, 2 pieces per thread
    (40, 50, 2500, 14, 0.5, np.float64),       # 512 threads, 1 piece
    (20, 30, 5000, 16, 1.0, np.float32),       # 512 threads, 2 pieces
    (33, 20, 9000, 13, 0.5, np.float64),       # 512 threads, 3 pieces
    (17, 19, 16384, 15, 2.0, np.float64),      # 512 threads, 4 pieces: the longest row it takes
    (18, 21, 16385, 12, 0.5, np.float64),      # one more: the kernel that reads a row twice
]


@pytest.mark.parametrize("m,n,k,N,phi,dtype", CASES)
def test_stage_parity(oz, oracle, m, n, k, N, phi, dtype):
    A, B = S.gemm_inputs(m, n, k, phi, seed=10 + N, dtype=dtype)
    is_double = dtype == np.float64
    ref = oracle.gemm(A, B, N, is_double=is_double)
    assert_parity(gpu_gemm(oz, A, B, N), ref, is_double)
    assert_parity(gpu_gemm(oz, A, B, N, int32_products=True, small_conversion=False), ref, is_double)


def test_k_beyond_2_pow_17_is_blocked(oz, oracle):
    """Section 4.3: k > 2^17 by block matrix multiplication; the residues of the K ranges are
    folded modulo p_s (compare U_s and C; the int32 planes are only congruent to C'_s)."""
    m, n, k = 64, 96, 2 ** 17 + 3 * 128 + 5
    A, B = S.gemm_inputs(m, n, k, 0.5, seed=7)
    ref = oracle.gemm(A, B, 14)
    got = gpu_gemm(oz, A, B, 14)
    assert_parity(got, ref, True)
    got = gpu_gemm(oz, A, B, 14, int32_products=True)
    p = np.array(ref["consts"].p)[:, None, None]
    assert np.array_equal(np.mod(got.pop("prod").astype(np.int64), p), ref["U"])
    assert_parity(got, ref, True)
    A32, B32 = A[:, :2 ** 17 + 128].astype(np.float32), B[:2 ** 17 + 128].astype(np.float32)
    assert_parity(gpu_gemm(oz, A32, B32, 8), oracle.gemm(A32, B32, 8, is_double=False), False)
    # accurate mode: Cbar in two K ranges, the sums of their maxima in place of the maxima
    assert_parity(gpu_gemm(oz, A, B, 14, accurate=True), oracle.gemm(A, B, 14, accurate=True), True)
    assert_parity(gpu_gemm(oz, A32, B32, 8, accurate=True),
                  oracle.gemm(A32, B32, 8, is_double=False, accurate=True), False)


def test_longest_contraction_k_2_pow_20(oz, oracle):
    """The largest k the fast mode takes (the exact integer sum of squares needs k 2^32 < 2^53):
    eight K ranges of 2^17, rows of A a million elements long, N = 20; one element more is
    refused."""
    import torch
    m, n, k = 20, 24, 2 ** 20
    A, B = S.gemm_inputs(m, n, k, 1.0, seed=8)
    A[3, :] = np.ldexp(np.sign(A[3, :]) + (A[3, :] == 0), 17)     # a row of +-2^17: the largest sum of squares
    assert_parity(gpu_gemm(oz, A, B, 20), oracle.gemm(A, B, 20), True)
    A32, B32 = A.astype(np.float32), B.astype(np.float32)
    assert_parity(gpu_gemm(oz, A32, B32, 9), oracle.gemm(A32, B32, 9, is_double=False), False)
    # accurate mode over eight K ranges; the row of +-2^17 makes 7-bit magnitudes of 32 throughout
    assert_parity(gpu_gemm(oz, A, B, 18, accurate=True), oracle.gemm(A, B, 18, accurate=True), True)
    dA = torch.zeros((2, k + 1), dtype=torch.float64, device="cuda")
    dB = torch.zeros((k + 1, 2), dtype=torch.float64, device="cuda")
    with pytest.raises(oz.OZ2Error) as e:
        oz.matmul(dA, dB, 14)
    assert e.value.status == 2


ACCURATE_CASES = [
    (256, 256, 256, 14, 0.5, np.float64),
    (1, 1, 1, 2, 0.5, np.float64),
    (300, 200, 333, 16, 2.0, np.float64),
    (520, 390, 1000, 12, 4.0, np.float64),
    (257, 513, 129, 20, 1.0, np.float64),
    (300, 200, 333, 7, 1.5, np.float32),
    (97, 515, 1030, 9, 0.5, np.float32),
]


@pytest.mark.parametrize("m,n,k,N,phi,dtype", ACCURATE_CASES)
def test_stage_parity_accurate_mode(oz, oracle, m, n, k, N, phi, dtype):
    A, B = S.gemm_inputs(m, n, k, phi, seed=30 + N, dtype=dtype)
    is_double = dtype == np.float64
    ref = oracle.gemm(A, B, N, is_double=is_double, accurate=True)
    assert_parity(gpu_gemm(oz, A, B, N, accurate=True), ref, is_double)
    assert_parity(gpu_gemm(oz, A, B, N, accurate=True, small_conversion=False), ref, is_double)


def test_accurate_mode_degenerate_inputs(oz, oracle):
    A, B = S.gemm_inputs(40, 50, 60, 1.0, seed=9)
    A[3, :] = 0.0; B[:, 7] = 0.0
    A[5, :] *= 2.0 ** -1040; B[:, 9] *= 2.0 ** 900
    A[7, :] = 1.0; B[:, 11] = -1.0
    Cin = S.matrix(40, 50, 0.5, seed=2)
    assert_parity(gpu_gemm(oz, A, B, 16, 0.5, 2.0, Cin.copy(), lda=77, ldb=64, accurate=True),
                  oracle.gemm(A, B, 16, 0.5, 2.0, Cin, accurate=True), True)
    assert_parity(gpu_gemm(oz, A, B, 16, 0.5, 2.0, Cin.copy(), lda=77, ldb=64, accurate=True,
                           small_conversion=False),
                  oracle.gemm(A, B, 16, 0.5, 2.0, Cin, accurate=True), True)
    Zb = np.zeros((60, 50))                      # B = 0: every maximum of Cbar is 0
    assert_parity(gpu_gemm(oz, A, Zb, 14, accurate=True), oracle.gemm(A, Zb, 14, accurate=True), True)
    assert_parity(gpu_gemm(oz, A, Zb, 14, accurate=True, small_conversion=False),
                  oracle.gemm(A, Zb, 14, accurate=True), True)


@pytest.mark.parametrize("N", [10, 11, 12, 13])
def test_accurate_mode_largest_scaled_integers(oz, oracle, N):
    """Accurate mode's scaled integers are largest when the maxima of Cbar are smallest: B = 0
    (maxima 0, taken as 1) and B with a single tiny entry per column.  Around 11-12 moduli they
    exceed what one round of the floating-point reduction handles (fast mode's never do there), so
    the residues of A must still be the symmetric ones."""
    A, B = S.gemm_inputs(70, 40, 200, 1.0, seed=40 + N)
    A = np.trunc(A * 2.0 ** 20) + 0.5 * np.sign(A)       # many low bits set after scaling
    Zb = np.zeros_like(B)
    for small in (True, False):
        assert_parity(gpu_gemm(oz, A, Zb, N, accurate=True, small_conversion=small),
                      oracle.gemm(A, Zb, N, accurate=True), True)
    B1 = np.zeros_like(B)
    B1[np.arange(40) % 200, np.arange(40)] = 2.0 ** -30 * (1 + np.arange(40))
    for small in (True, False):
        assert_parity(gpu_gemm(oz, A, B1, N, accurate=True, small_conversion=small),
                      oracle.gemm(A, B1, N, accurate=True), True)


def test_alpha_beta_and_leading_dimensions(oz, oracle):
    A, B = S.gemm_inputs(70, 90, 150, 0.5, seed=3)
    Cin = S.matrix(70, 90, 0.5, seed=5)
    for alpha, beta in ((1.0, 0.0), (-2.5, 0.0), (1.0, 1.0), (0.75, -0.5), (0.0, 2.0)):
        ref = oracle.gemm(A, B, 15, alpha, beta, Cin)
        got = gpu_gemm(oz, A, B, 15, alpha, beta, Cin.copy(), lda=160, ldb=97)
        assert_parity(got, ref, True)
    A32, B32, C32 = A.astype(np.float32), B.astype(np.float32), Cin.astype(np.float32)
    ref = oracle.gemm(A32, B32, 8, 1.5, 0.25, C32, is_double=False)
    got = gpu_gemm(oz, A32, B32, 8, 1.5, 0.25, C32.copy(), lda=151, ldb=128)
    assert_parity(got, ref, False)


def test_unaligned_operands_and_strided_c(oz, oracle):
    """Pointers and leading dimensions that defeat the 16-byte fast paths of the kernels."""
    import torch
    A, B = S.gemm_inputs(37, 53, 100, 0.5, seed=12)
    ref = oracle.gemm(A, B, 14)
    assert_parity(gpu_gemm(oz, A, B, 14, lda=101, ldb=59, ldc=61, c_offset=1), ref, True)
    assert_parity(gpu_gemm(oz, A, B, 14, ldc=64, c_offset=2), ref, True)
    A32, B32 = A.astype(np.float32), B.astype(np.float32)
    ref = oracle.gemm(A32, B32, 8, is_double=False)
    assert_parity(gpu_gemm(oz, A32, B32, 8, lda=103, ldb=55, ldc=57, c_offset=3), ref, False)
    # A and B that start at odd element offsets
    dt = torch.float64
    sa = torch.zeros(37 * 100 + 1, dtype=dt, device="cuda"); sb = torch.zeros(100 * 53 + 1, dtype=dt, device="cuda")
    dA = sa[1:].view(37, 100); dB = sb[1:].view(100, 53)
    dA.copy_(torch.from_numpy(A).cuda()); dB.copy_(torch.from_numpy(B).cuda())
    C = oz.matmul(dA, dB, 14)
    assert np.array_equal(C.cpu().numpy(), oracle.gemm(A, B, 14)["C"])


def test_large_tile_kernel_without_the_xcd_swizzle(oz, oracle):
    """6 x 5 tiles of 256: the 8-wavefront kernel with the plain tile map (the swizzled map
    needs multiples of 16 tiles), ragged edges, both product forms."""
    A, B = S.gemm_inputs(1300, 1100, 300, 1.0, seed=13)
    ref = oracle.gemm(A, B, 20)
    assert_parity(gpu_gemm(oz, A, B, 20), ref, True)
    assert_parity(gpu_gemm(oz, A, B, 20, int32_products=True), ref, True)


def test_beta_zero_does_not_read_c(oz, oracle):
    A, B = S.gemm_inputs(33, 17, 40, 0.5, seed=1)
    got = gpu_gemm(oz, A, B, 14, 2.0, 0.0, np.full((33, 17), np.nan))
    assert_parity(got, oracle.gemm(A, B, 14, 2.0, 0.0), True)


def test_degenerate_inputs(oz, oracle):
    A, B = S.gemm_inputs(40, 50, 60, 1.0, seed=9)
    A[3, :] = 0.0                       # zero row
    B[:, 7] = 0.0                       # zero column
    A[5, :] *= 2.0 ** -1040             # subnormal row
    B[:, 9] *= 2.0 ** 900               # huge column
    A[6, :] = 0.0; A[6, 11] = -1.0      # single entry
    A[7, :] = 1.0                       # constant rows and columns: worst case of the bound
    B[:, 11] = -1.0
    ref = oracle.gemm(A, B, 16)
    assert_parity(gpu_gemm(oz, A, B, 16), ref, True)
    assert_parity(gpu_gemm(oz, A, B, 16, small_conversion=False), ref, True)        # the general kernels
    Z = np.zeros((20, 30)); Zb = np.zeros((30, 10))
    assert_parity(gpu_gemm(oz, Z, Zb, 14), oracle.gemm(Z, Zb, 14), True)
    assert_parity(gpu_gemm(oz, Z, Zb, 14, small_conversion=False), oracle.gemm(Z, Zb, 14), True)


def test_nonfinite_inputs_stay_local_and_memory_safe(oz, oracle):
    """Inf/NaN inputs are outside the method (the result in their row / column is unspecified)
    but must not disturb anything else: shifts are per row of A and per column of B."""
    A, B = S.gemm_inputs(48, 40, 70, 0.5, seed=14)
    A_bad, B_bad = A.copy(), B.copy()
    A_bad[5, 3] = np.nan; A_bad[9, 0] = np.inf; B_bad[7, 11] = -np.inf; B_bad[0, 2] = np.nan
    ref = oracle.gemm(A, B, 15)["C"]
    rows = np.setdiff1d(np.arange(48), [5, 9]); cols = np.setdiff1d(np.arange(40), [11, 2])
    for small in (True, False):                  # fast mode only: accurate mode couples rows through Cbar's maxima
        got = gpu_gemm(oz, A_bad, B_bad, 15, small_conversion=small)["C"]
        assert np.array_equal(got[np.ix_(rows, cols)], ref[np.ix_(rows, cols)])
        gpu_gemm(oz, A_bad, B_bad, 15, accurate=True, small_conversion=small)    # must simply return


def test_empty_and_k_zero(oz):
    import torch
    C = torch.full((4, 5), 3.0, dtype=torch.float64, device="cuda")
    A = torch.zeros((4, 1), dtype=torch.float64, device="cuda")
    oz.oz2_dgemm(0, 5, 3, 1.0, A, 3, A, 5, 0.0, C, 5, 14)
    oz.oz2_dgemm(4, 0, 3, 1.0, A, 3, A, 1, 0.0, C, 1, 14)
    torch.cuda.synchronize()
    assert bool((C == 3.0).all())
    oz.oz2_dgemm(4, 5, 0, 1.0, A, 1, A, 5, 0.5, C, 5, 14)      # k = 0: C <- beta C
    torch.cuda.synchronize()
    assert bool((C == 1.5).all())
    oz.oz2_dgemm(4, 5, 0, 1.0, A, 1, A, 5, 0.0, C, 5, 14)
    torch.cuda.synchronize()
    assert bool((C == 0.0).all())


def test_mfma_probe_reports_a_plausible_rate(oz):
    # the matrix cores alone: below the published dense INT8 peak (5.0e15 op/s, with a margin
    # for a boost above the nominal clock) and far above anything the vector ALUs could do
    import torch
    for random_operands in (False, True):
        tops, cus, mhz = oz.oz2_mfma_probe(random_operands, 0.05)
        assert cus == torch.cuda.get_device_properties(0).multi_processor_count
        assert 500.0 < tops < 5600.0 and mhz > 0


def test_int8_gemm_random_and_extreme(oz, oracle):
    import torch
    rng = np.random.default_rng(0)
    batch, Mp, Np, Kp = 3, 256, 512, 384
    A = rng.integers(-128, 128, (batch, Mp, Kp), dtype=np.int8)
    B = rng.integers(-128, 128, (batch, Np, Kp), dtype=np.int8)
    A[0, :7, :] = -128; B[0, :9, :] = -128; A[1, 3, :] = 127; B[1, 5, :] = 127
    dC = torch.empty((batch, Mp, Np), dtype=torch.int32, device="cuda")
    oz.oz2_int8_gemm(oz.block_slices(torch.from_numpy(A).cuda()),
                     oz.block_slices(torch.from_numpy(B).cuda()), dC, batch, Mp, Np, Kp)
    ref = oracle.int8_gemm_rows(A, B, np.arange(Mp))
    assert np.array_equal(dC.cpu().numpy(), ref)


def test_int32_wrap_at_k_2_pow_17(oz):
    """Section 4.3: k = 2^17 with all residues -128 sums to 2^31, which wraps to -2^31."""
    import torch
    Mp = Np = 256; Kp = 2 ** 17
    A = torch.full((1, Mp, Kp), -128, dtype=torch.int8, device="cuda")
    A[0, 1, :] = 127
    A[0, 2, -1] = 0
    C = torch.empty((1, Mp, Np), dtype=torch.int32, device="cuda")
    A = oz.block_slices(A)
    oz.oz2_int8_gemm(A, A, C, 1, Mp, Np, Kp)
    c = C.cpu().numpy()[0]
    assert c[0, 0] == -2 ** 31 and c[5, 9] == -2 ** 31
    assert c[1, 1] == 127 * 127 * Kp and c[0, 1] == -128 * 127 * Kp
    assert c[2, 2] == 2 ** 31 - 128 * 128 and c[0, 2] == 2 ** 31 - 128 * 128


def test_determinism(oz):
    import torch
    A, B = S.gemm_inputs(300, 280, 500, 0.5, seed=4)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    c1 = oz.matmul(dA, dB, 15).clone()
    c2 = oz.matmul(dA, dB, 15)
    assert torch.equal(c1, c2)


def test_caller_owned_workspace(oz, oracle):
    import torch
    A, B = S.gemm_inputs(100, 120, 140, 0.5, seed=6)
    need = oz.oz2_workspace_bytes(100, 120, 140, 14, True)
    least = oz.oz2_workspace_min_bytes(100, 120, 140, 14, True)
    assert least == need                                   # C fits one 256 x 256 panel
    small = torch.empty(least - 256, dtype=torch.uint8, device="cuda")
    oz.oz2_set_workspace(small)
    with pytest.raises(oz.OZ2Error) as e:
        oz.matmul(torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda(), 14)
    assert e.value.status == 3
    buf = torch.empty(need, dtype=torch.uint8, device="cuda")
    oz.oz2_set_workspace(buf)
    try:
        assert_parity(gpu_gemm(oz, A, B, 14), oracle.gemm(A, B, 14), True)
    finally:
        oz.oz2_set_workspace(None)


# ------------------------------------------------------------------ benchmark-size configurations
def band_rows(m, rng, band=256):
    """One row out of every `band` consecutive rows (every row of tiles of the INT8 GEMM is hit),
    plus the first and the last row."""
    starts = np.arange(0, m, band)
    picks = starts + rng.integers(0, np.minimum(band, m - starts))
    return np.unique(np.concatenate([[0, m - 1], picks]))


def sampled_parity(oz, oracle, m, n, k, N, phi, dtype, seed, n_rows=6, n_entries=1500,
                   accurate=False, int32_products=False, inputs=None, bands=None):
    """Full comparison of shifts and residues, sampled comparison of products and C.
    inputs: (A, B, dA, dB) generated before (several N on one pair of matrices);
    bands: compare one full row per `bands` rows instead of n_rows random ones."""
    import torch
    from paper_2508_03984_amd import binding as b
    is_double = dtype == np.float64
    print(f"sampled parity: {m} x {n} x {k}, N = {N}, phi = {phi}, {np.dtype(dtype).name}, "
          f"accurate = {accurate}", flush=True)
    if inputs is None:
        A, B = S.gemm_inputs(m, n, k, phi, seed, dtype)
        dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    else:
        A, B, dA, dB = inputs
    # the overlapped form (an option; it applies above 4096 x 4096 with a long k) first, then the
    # default form, everything on one stream, which keeps the products of all of C for the checks
    # below; the two must agree bit for bit
    oz.oz2_set_overlap(True)
    try:
        dC_overlapped = oz.matmul(dA, dB, N, accurate=accurate)
    finally:
        oz.oz2_set_overlap(False)
    oz.oz2_set_int32_products(int32_products)
    try:
        dC = oz.matmul(dA, dB, N, accurate=accurate)
    finally:
        oz.oz2_set_int32_products(False)
    torch.cuda.synchronize()
    assert torch.equal(dC_overlapped, dC), "overlapped and single-stream results differ"
    del dC_overlapped
    prep = oracle.prepare(A, B, N, is_double, accurate)
    assert np.array_equal(oz.stage_tensor(b.OZ2_STAGE_SHIFT_A).cpu().numpy(), prep["tA"])
    assert np.array_equal(oz.stage_tensor(b.OZ2_STAGE_SHIFT_B).cpu().numpy(), prep["tB"])
    ra = oz.unblock_slices(oz.stage_tensor(b.OZ2_STAGE_RES_A, copy=False))    # a permuted view
    for s in range(N):                                   # compare on the device, slice by slice
        assert torch.equal(ra[s, :m, :k], torch.from_numpy(prep["Ares"][s]).cuda()), f"A slice {s}"
    del ra
    rb = oz.unblock_slices(oz.stage_tensor(b.OZ2_STAGE_RES_B, copy=False))
    for s in range(N):
        assert torch.equal(rb[s, :n, :k], torch.from_numpy(prep["Bres"][s]).cuda()), f"B slice {s}"
    del rb
    rng = np.random.default_rng(seed)
    if bands:
        rows = band_rows(m, rng, bands)
    else:
        rows = np.unique(np.concatenate([[0, m - 1], rng.integers(0, m, n_rows)]))
    fin = oracle.finish_rows(prep, rows)
    stage, key = (b.OZ2_STAGE_PROD, "prod") if int32_products else (b.OZ2_STAGE_U, "U")
    prod = oz.stage_tensor(stage, copy=False)
    got_rows = prod[:, torch.from_numpy(rows).cuda(), :n].cpu().numpy()
    assert np.array_equal(got_rows, fin[key]), f"{key} differs on sampled rows"
    ii = rng.integers(0, m, n_entries); jj = rng.integers(0, n, n_entries)
    ent = oracle.finish_entries(prep, ii, jj)
    ti, tj = torch.from_numpy(ii).cuda(), torch.from_numpy(jj).cuda()
    assert np.array_equal(prod[:, ti, tj].cpu().numpy(), ent[key])
    del prod
    tol = TOL64 if is_double else TOL32
    for got, ref in ((dC[torch.from_numpy(rows).cuda()].cpu().numpy(), fin["C"]),
                     (dC[ti, tj].cpu().numpy(), ent["C"])):
        g, r = got.astype(np.float64), ref.astype(np.float64)
        assert np.max(np.abs(g - r) / np.where(r == 0, 1.0, np.abs(r))) <= tol
    return dC


def device_inputs(m, n, k, phi, seed, dtype):
    import torch
    A, B = S.gemm_inputs(m, n, k, phi, seed, dtype)
    return A, B, torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()


def test_config_4096_sampled(oz, oracle):
    for N in (12, 16, 20):
        sampled_parity(oz, oracle, 4096, 4096, 4096, N, 0.5, np.float64, seed=0)
    sampled_parity(oz, oracle, 4096, 4096, 4096, 14, 0.5, np.float64, seed=0, int32_products=True)


def test_config_4096_accurate_sampled(oz, oracle):
    sampled_parity(oz, oracle, 4096, 4096, 4096, 15, 2.0, np.float64, seed=0, accurate=True)


def test_config_16384_dgemm_sampled(oz, oracle):
    """The headline configuration: shifts and residues in full; products and C on one full row out
    of every 256 (66 rows: every row of output tiles, and with all columns every tile of every
    modulus) and on 10^5 scattered entries."""
    sampled_parity(oz, oracle, 16384, 16384, 16384, 16, 0.5, np.float64, seed=0,
                   bands=256, n_entries=100000)
    assert oz.oz2_last_panels() == (16384, 16384, 1) and oz.oz2_last_gemm_launches() == 8


def test_gemm_launches_cut_in_place(oz, oracle):
    """A product whose planes all fit the workspace runs its INT8 GEMMs as several launches for a
    long contraction (here 4096 + 512 rows by 8192 + 512 columns: four launches, ragged ones
    included), each writing its part of the whole product in place: products and C equal the
    oracle's on rows of every launch panel; a short contraction stays one launch."""
    sampled_parity(oz, oracle, 4500, 8600, 8200, 6, 1.0, np.float64, seed=31, bands=512, n_entries=4000)
    assert oz.oz2_last_panels() == (4608, 8704, 1) and oz.oz2_last_gemm_launches() == 4
    sampled_parity(oz, oracle, 4500, 8600, 520, 14, 0.5, np.float64, seed=32, n_rows=4, n_entries=1000)
    assert oz.oz2_last_panels() == (4608, 8704, 1) and oz.oz2_last_gemm_launches() == 1
    # the option that switches the cut off: one launch, the same bits
    import torch
    from paper_2508_03984_amd import binding as b
    A, B, dA, dB = device_inputs(4500, 8600, 8200, 1.0, 31, np.float64)
    cut = oz.matmul(dA, dB, 6)
    assert oz.oz2_last_gemm_launches() == 4
    oz.oz2_ctx_set_option(None, b.OZ2_OPT_CUT_LAUNCHES, False)
    try:
        whole = oz.matmul(dA, dB, 6)
        assert oz.oz2_last_gemm_launches() == 1
    finally:
        oz.oz2_ctx_set_option(None, b.OZ2_OPT_CUT_LAUNCHES, True)
    assert torch.equal(cut, whole)
    oz.oz2_release()


def test_gemm_launches_cut_along_k(oz, oracle):
    """Launches with many rounds of workgroups and a long contraction are also cut along k (here two
    K ranges of 24576 although k < 2^17): the second range is folded onto the first modulo p_s in
    the store phase, and U_s and C still equal the oracle's."""
    sampled_parity(oz, oracle, 4096, 4096, 49152, 16, 0.5, np.float64, seed=33, n_rows=3, n_entries=3000)
    assert oz.oz2_last_panels() == (4096, 4096, 1) and oz.oz2_last_gemm_launches() == 2
    oz.oz2_release()


@pytest.mark.parametrize("phi,N", [(1.0, 18), (2.0, 20)])
def test_config_16384_dgemm_wider_exponent_range_sampled(oz, oracle, phi, N):
    """The other corners of the 16384^3 configuration (phi up to 2, up to 20 moduli, the widest
    scaled integers): one row per 1024 rows and 20000 entries."""
    sampled_parity(oz, oracle, 16384, 16384, 16384, N, phi, np.float64, seed=0,
                   bands=1024, n_entries=20000)
    oz.oz2_release()


def test_config_sgemm_8192_sampled(oz, oracle):
    inputs = device_inputs(8192, 8192, 8192, 0.5, 0, np.float32)
    for N in (5, 8, 9):                           # the moduli counts of Section 5.2's SGEMM figures
        sampled_parity(oz, oracle, 8192, 8192, 8192, N, 0.5, np.float32, seed=0, bands=1024,
                       n_entries=5000, inputs=inputs)


def test_config_sgemm_16384_sampled(oz, oracle):
    inputs = device_inputs(16384, 16384, 16384, 0.5, 0, np.float32)
    for N in (5, 8, 9):
        sampled_parity(oz, oracle, 16384, 16384, 16384, N, 0.5, np.float32, seed=0, bands=1024,
                       n_entries=20000, inputs=inputs)
    oz.oz2_release()


def test_config_nonsquare_k_65536_sampled(oz, oracle):
    sampled_parity(oz, oracle, 8192, 8192, 65536, 18, 1.0, np.float64, seed=0,
                   n_rows=2, n_entries=500)


def test_large_and_skewed_shapes_sampled(oz, oracle):
    """Shapes far from the benchmark's: 2^30 entries of C (index arithmetic beyond 32 bits),
    a tall and a wide product, one in accurate mode, one in FP32."""
    sampled_parity(oz, oracle, 32768, 32768, 2048, 16, 0.5, np.float64, seed=3, n_rows=2, n_entries=500)
    sampled_parity(oz, oracle, 40000, 300, 4096, 15, 1.0, np.float64, seed=4, n_rows=2, n_entries=500,
                   accurate=True)
    sampled_parity(oz, oracle, 300, 50000, 1000, 8, 1.0, np.float32, seed=5, n_rows=2, n_entries=500)
    oz.oz2_release()


def test_short_contractions_use_the_persistent_gemm(oz, oracle):
    """k <= 4096 with at least 128 large tiles runs the persistent form of the INT8 GEMM (every
    workgroup walks over several tiles): full parity on a ragged shape in both product forms,
    and the folding store phases (second K range of a k > 2^17 product, 428 deep) on samples."""
    A, B = S.gemm_inputs(1100, 1500, 700, 1.0, seed=21)             # 5 x 6 tiles x 16 moduli
    ref = oracle.gemm(A, B, 16)
    assert_parity(gpu_gemm(oz, A, B, 16), ref, True)
    assert_parity(gpu_gemm(oz, A, B, 16, int32_products=True), ref, True)
    A32, B32 = S.gemm_inputs(3000, 2100, 1024, 0.5, seed=22, dtype=np.float32)   # 12 x 9 tiles x 8
    assert_parity(gpu_gemm(oz, A32, B32, 8), oracle.gemm(A32, B32, 8, is_double=False), False)
    sampled_parity(oz, oracle, 1536, 1536, 2 ** 17 + 300, 4, 0.5, np.float32, seed=23, n_rows=2, n_entries=300)
    oz.oz2_release()


def test_int8_gemm_persistent_form_direct(oz, oracle):
    """oz2_int8_gemm on a shape that takes the persistent kernel (192 large tiles, K = 512, not a
    multiple of 16 tiles: plain tile map), INT32 output, against the oracle on sampled rows."""
    import torch
    rng = np.random.default_rng(7)
    batch, Mp, Np, Kp = 4, 1536, 2048, 512
    A = rng.integers(-128, 128, (batch, Mp, Kp), dtype=np.int8)
    B = rng.integers(-128, 128, (batch, Np, Kp), dtype=np.int8)
    dC = torch.empty((batch, Mp, Np), dtype=torch.int32, device="cuda")
    oz.oz2_int8_gemm(oz.block_slices(torch.from_numpy(A).cuda()),
                     oz.block_slices(torch.from_numpy(B).cuda()), dC, batch, Mp, Np, Kp)
    rows = np.array([0, 255, 256, 700, 1279, 1535])
    ref = oracle.int8_gemm_rows(A, B, rows)
    assert np.array_equal(dC[:, torch.from_numpy(rows).cuda(), :].cpu().numpy(), ref)
