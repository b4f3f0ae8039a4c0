"""GPU parity of the general entry points: transposed operands (oz2_*gemm_op), prepared
operands (oz2_prepare_* / oz2_*gemm_prepared) and products cut into panels by a bounded
workspace.  The oracle knows none of these: a transposed operand is handed to it as the matrix
it stands for, and a panelled or prepared product must equal the plain one bit for bit."""
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
    oz.load()
    yield oz
    oz.oz2_set_workspace_limit(0)
    oz.oz2_release()


@pytest.fixture(autouse=True)
def overlap_option_for_the_overlapped_tests(request, oz):
    """The overlapped form is an option (off by default): the tests about it switch it on."""
    on = "overlapped" in request.node.name
    if on:
        oz.oz2_set_overlap(True)
    yield
    if on:
        oz.oz2_set_overlap(False)


def stored(X, transposed, ld_extra, dt):
    """X (numpy) on the device as op(stored): stored = X or X^T, rows padded by ld_extra."""
    import torch
    M = np.ascontiguousarray(X.T) if transposed else X
    buf = torch.full((M.shape[0], M.shape[1] + ld_extra), 7.0, dtype=dt, device="cuda")
    buf[:, :M.shape[1]] = torch.from_numpy(M).cuda()
    return buf, M.shape[1] + ld_extra


def run_op(oz, A, B, N, opA, opB, accurate=False, alpha=1.0, beta=0.0, Cin=None, lda_extra=3, ldb_extra=5,
           small_conversion=True):
    import torch
    from paper_2508_03984_amd import binding as b
    m, k = A.shape
    n = B.shape[1]
    is_double = A.dtype == np.float64
    dt = torch.float64 if is_double else torch.float32
    dA, lda = stored(A, opA, lda_extra, dt)
    dB, ldb = stored(B, opB, ldb_extra, dt)
    dC = torch.full((m, n), float("nan"), dtype=dt, device="cuda")
    if Cin is not None:
        dC.copy_(torch.from_numpy(Cin).cuda())
    fn = oz.oz2_dgemm_op if is_double else oz.oz2_sgemm_op
    oz.oz2_set_small_conversion(small_conversion)
    try:
        fn(int(opA), int(opB), accurate, m, n, k, alpha, dA, lda, dB, ldb, beta, dC, n, N)
    finally:
        oz.oz2_set_small_conversion(True)
    torch.cuda.synchronize()
    ra = oz.unblock_slices(oz.stage_tensor(b.OZ2_STAGE_RES_A))
    rb = oz.unblock_slices(oz.stage_tensor(b.OZ2_STAGE_RES_B))
    assert bool((ra[:, m:, :] == 0).all() and (ra[:, :, k:] == 0).all())
    assert bool((rb[:, n:, :] == 0).all() and (rb[:, :, k:] == 0).all())
    return dict(C=dC.cpu().numpy(), tA=oz.stage_tensor(b.OZ2_STAGE_SHIFT_A).cpu().numpy(),
                tB=oz.stage_tensor(b.OZ2_STAGE_SHIFT_B).cpu().numpy(),
                Ares=ra[:, :m, :k].cpu().numpy(), Bres=rb[:, :n, :k].cpu().numpy(),
                U=oz.stage_tensor(b.OZ2_STAGE_U)[:, :m, :n].cpu().numpy())


def check(got, ref, is_double):
    for key in ("tA", "tB", "Ares", "Bres", "U"):
        assert np.array_equal(got[key], ref[key]), key
    c, r = got["C"].astype(np.float64), ref["C"].astype(np.float64)
    rel = np.max(np.abs(c - r) / np.where(r == 0, 1.0, np.abs(r)))
    assert rel <= (TOL64 if is_double else TOL32), rel


OP_CASES = [
    # m, n, k, N, phi, dtype
    (300, 200, 333, 16, 0.5, np.float64),
    (70, 130, 515, 13, 2.0, np.float64),
    (1, 1, 1, 2, 0.5, np.float64),
    (257, 65, 129, 20, 1.0, np.float64),
    (300, 200, 333, 8, 0.5, np.float32),
    (97, 515, 260, 5, 1.0, np.float32),
]


@pytest.mark.parametrize("opA,opB", [(0, 1), (1, 0), (1, 1), (0, 0)])
@pytest.mark.parametrize("m,n,k,N,phi,dtype", OP_CASES)
def test_transposed_operands_fast_mode(oz, oracle, m, n, k, N, phi, dtype, opA, opB):
    A, B = S.gemm_inputs(m, n, k, phi, seed=50 + N, dtype=dtype)
    is_double = dtype == np.float64
    ref = oracle.gemm(A, B, N, is_double=is_double)
    check(run_op(oz, A, B, N, opA, opB), ref, is_double)
    check(run_op(oz, A, B, N, opA, opB, small_conversion=False), ref, is_double)    # the general kernels


@pytest.mark.parametrize("opA,opB", [(0, 1), (1, 0), (1, 1)])
def test_transposed_operands_accurate_mode_alpha_beta(oz, oracle, opA, opB):
    A, B = S.gemm_inputs(150, 260, 300, 2.0, seed=61)
    A[4, :] = 0.0; B[:, 9] = 0.0
    Cin = S.matrix(150, 260, 0.5, seed=62)
    ref = oracle.gemm(A, B, 15, -0.75, 1.5, Cin, accurate=True)
    check(run_op(oz, A, B, 15, opA, opB, True, -0.75, 1.5, Cin), ref, True)
    check(run_op(oz, A, B, 15, opA, opB, True, -0.75, 1.5, Cin, small_conversion=False), ref, True)
    A32, B32 = A.astype(np.float32), B.astype(np.float32)
    ref = oracle.gemm(A32, B32, 7, is_double=False, accurate=True)
    check(run_op(oz, A32, B32, 7, opA, opB, True), ref, False)


def test_matmul_accepts_transposed_views(oz, oracle):
    import torch
    A, B = S.gemm_inputs(90, 70, 110, 0.5, seed=63)
    want = oracle.gemm(A, B, 14)["C"]
    dAt = torch.from_numpy(np.ascontiguousarray(A.T)).cuda()
    dBt = torch.from_numpy(np.ascontiguousarray(B.T)).cuda()
    assert np.array_equal(oz.matmul(dAt.t(), dBt.t(), 14).cpu().numpy(), want)
    assert np.array_equal(oz.matmul(torch.from_numpy(A).cuda(), dBt.t(), 14).cpu().numpy(), want)
    # the Gram matrix A A^T from one stored matrix
    dA = torch.from_numpy(A).cuda()
    assert np.array_equal(oz.matmul(dA, dA.t(), 14).cpu().numpy(),
                          oracle.gemm(A, np.ascontiguousarray(A.T), 14)["C"])


def test_op_argument_checks(oz):
    import torch
    X = torch.zeros((8, 8), dtype=torch.float64, device="cuda")
    for bad in (dict(opA=2), dict(opB=-1), dict(lda=3), dict(ldb=3)):
        a = dict(opA=1, opB=0, lda=4, ldb=6)
        a.update(bad)
        with pytest.raises(oz.OZ2Error) as e:               # op(A) = A^T: stored 5 x 4, lda >= 4
            oz.oz2_dgemm_op(a["opA"], a["opB"], 0, 4, 6, 5, 1.0, X, a["lda"], X, a["ldb"], 0.0, X, 8, 14)
        assert e.value.status == 1


@pytest.mark.parametrize("dtype,N,accurate", [(np.float64, 15, False), (np.float64, 14, True), (np.float32, 7, False)])
def test_column_major_entry_points(oz, oracle, dtype, N, accurate):
    """oz2_*gemm_colmajor: every matrix column-major, as a BLAS caller holds them.  A column-major
    array is built here as the row-major storage of the transpose; the result must equal the
    oracle's for the matrices the arrays stand for, in all four transposition cases."""
    import torch
    m, n, k = 150, 210, 333
    A, B = S.gemm_inputs(m, n, k, 1.0, seed=90 + N, dtype=dtype)
    Cin = S.matrix(m, n, 0.5, seed=91, dtype=dtype)
    is_double = dtype == np.float64
    ref = oracle.gemm(A, B, N, 0.5, -1.5, Cin, is_double=is_double, accurate=accurate)["C"]
    dt = torch.float64 if is_double else torch.float32
    fn = oz.oz2_dgemm_colmajor if is_double else oz.oz2_sgemm_colmajor

    def colmajor(X, extra):           # column-major X with leading dimension rows + extra
        buf = torch.full((X.shape[1], X.shape[0] + extra), 3.0, dtype=dt, device="cuda")
        buf[:, :X.shape[0]] = torch.from_numpy(np.ascontiguousarray(X.T)).cuda()
        return buf, X.shape[0] + extra

    for opA in (0, 1):
        for opB in (0, 1):
            dA, lda = colmajor(A.T if opA else A, 3)          # op = T: the stored matrix is the transpose
            dB, ldb = colmajor(B.T if opB else B, 1)
            dC, ldc = colmajor(Cin, 2)
            fn(opA, opB, accurate, m, n, k, 0.5, dA, lda, dB, ldb, -1.5, dC, ldc, N)
            torch.cuda.synchronize()
            got = dC[:, :m].t().cpu().numpy().astype(np.float64)
            r = ref.astype(np.float64)
            rel = np.max(np.abs(got - r) / np.where(r == 0, 1.0, np.abs(r)))
            assert rel <= (TOL64 if is_double else TOL32), (opA, opB, rel)
            assert bool((dC[:, m:] == 3.0).all())             # the gap between columns is untouched


# ------------------------------------------------------------------ bounded workspace
@pytest.mark.parametrize("accurate", [False, True])
@pytest.mark.parametrize("dtype,N", [(np.float64, 15), (np.float32, 6)])
def test_panelled_product_is_bit_identical(oz, oracle, dtype, N, accurate):
    import torch
    m, n, k = 700, 1100, 200                               # 3 x 5 tiles of 256
    A, B = S.gemm_inputs(m, n, k, 1.0, seed=70, dtype=dtype)
    Cin = S.matrix(m, n, 0.5, seed=71, dtype=dtype)
    is_double = dtype == np.float64
    ref = oracle.gemm(A, B, N, 0.5, -2.0, Cin, is_double=is_double, accurate=accurate)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    whole = oz.matmul(dA, dB, N, 0.5, -2.0, torch.from_numpy(Cin).cuda(), accurate=accurate)
    assert oz.oz2_last_panels() == (768, 1280, 1)
    need = oz.oz2_workspace_bytes(m, n, k, N, is_double)
    least = oz.oz2_workspace_min_bytes(m, n, k, N, is_double)
    per_entry = N
    seen = set()
    try:
        for entries in (256 * 256, 2 * 256 * 256, 512 * 512 + 7, 768 * 512, 768 * 1024 + 100):
            limit = least - 256 * 256 * per_entry + entries * per_entry
            assert limit < need
            oz.oz2_set_workspace_limit(limit)
            oz.oz2_release()                               # a buffer allocated earlier may be larger
            got = oz.matmul(dA, dB, N, 0.5, -2.0, torch.from_numpy(Cin).cuda(), accurate=accurate)
            pr, pc, count = oz.oz2_last_panels()
            assert (pr, pc, count) == oz.oz2_plan_panels(m, n, k, N, limit)
            assert count > 1 and pr * pc <= entries and pr % 256 == 0 and pc % 256 == 0
            seen.add((pr, pc))
            assert torch.equal(got, whole), (pr, pc)
            from paper_2508_03984_amd import binding as b
            assert np.array_equal(oz.stage_tensor(b.OZ2_STAGE_SHIFT_A).cpu().numpy(), ref["tA"])
            assert np.array_equal(oz.stage_tensor(b.OZ2_STAGE_SHIFT_B).cpu().numpy(), ref["tB"])
            with pytest.raises(oz.OZ2Error):               # only the last panel's products remain
                oz.oz2_stage_ptr(b.OZ2_STAGE_U)
        oz.oz2_set_workspace_limit(least - 256)
        oz.oz2_release()
        with pytest.raises(oz.OZ2Error) as e:
            oz.matmul(dA, dB, N)
        assert e.value.status == 3
    finally:
        oz.oz2_set_workspace_limit(0)
        oz.oz2_release()
    assert len(seen) >= 4                                  # different cuts were exercised
    c, r = whole.cpu().numpy().astype(np.float64), ref["C"].astype(np.float64)
    assert np.max(np.abs(c - r) / np.where(r == 0, 1.0, np.abs(r))) <= (TOL64 if is_double else TOL32)


def test_panelled_product_with_k_ranges_and_caller_workspace(oz, oracle):
    """k > 2^17 (two K ranges folded modulo p_s) inside each of several panels, in a
    caller-owned workspace that is too small for all of C."""
    import torch
    m, n, k = 260, 24, 2 ** 17 + 200
    A, B = S.gemm_inputs(m, n, k, 0.5, seed=72)
    ref = oracle.gemm(A, B, 14)
    least = oz.oz2_workspace_min_bytes(m, n, k, 14, True)
    buf = torch.empty(least, dtype=torch.uint8, device="cuda")     # one tile of C at a time
    oz.oz2_set_workspace(buf)
    try:
        got = oz.matmul(torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda(), 14)
        assert oz.oz2_last_panels() == (256, 256, 2)
        assert np.array_equal(got.cpu().numpy(), ref["C"])
    finally:
        oz.oz2_set_workspace(None)


# ------------------------------------------------------------------ prepared operands
@pytest.mark.parametrize("dtype,N", [(np.float64, 16), (np.float32, 8)])
def test_prepared_operands_equal_the_plain_call(oz, oracle, dtype, N):
    import torch
    m, n, k = 300, 200, 333
    is_double = dtype == np.float64
    dt = torch.float64 if is_double else torch.float32
    A, B = S.gemm_inputs(m, n, k, 0.5, seed=80, dtype=dtype)
    B2 = S.matrix(k, 90, 1.0, seed=82, dtype=dtype)
    Cin = S.matrix(m, n, 0.5, seed=81, dtype=dtype)
    prep = oz.oz2_prepare_d if is_double else oz.oz2_prepare_s
    prod = oz.oz2_dgemm_prepared if is_double else oz.oz2_sgemm_prepared
    tol = TOL64 if is_double else TOL32
    for opA in (0, 1):
        for opB in (0, 1):
            dA, lda = stored(A, opA, 2, dt)
            dB, ldb = stored(B, opB, 1, dt)
            L = prep(0, opA, m, k, dA, lda, N)
            R = prep(1, opB, n, k, dB, ldb, N)
            assert L.nbytes >= N * 512 * 384 and R.nbytes >= N * 256 * 384
            dA.fill_(1.0); dB.fill_(1.0)                   # the operands hold everything needed
            dC = torch.from_numpy(Cin).cuda()
            prod(L, R, 1.5, 0.25, dC, n)
            want = oracle.gemm(A, B, N, 1.5, 0.25, Cin, is_double=is_double)["C"]
            c, r = dC.cpu().numpy().astype(np.float64), want.astype(np.float64)
            assert np.max(np.abs(c - r) / np.where(r == 0, 1.0, np.abs(r))) <= tol
            # the left operand again, with another right factor
            dB2, ldb2 = stored(B2, opB, 0, dt)
            R2 = prep(1, opB, 90, k, dB2, ldb2, N)
            dC2 = torch.empty((m, 90), dtype=dt, device="cuda")
            prod(L, R2, 1.0, 0.0, dC2, 90)
            assert np.array_equal(dC2.cpu().numpy(), oracle.gemm(A, B2, N, is_double=is_double)["C"])
            with pytest.raises(oz.OZ2Error):               # no stage of a prepared product is kept
                oz.oz2_stage_ptr(0)
            for h in (L, R, R2):
                h.free()


def test_prepared_operand_checks(oz):
    import torch
    X = torch.zeros((300, 300), dtype=torch.float64, device="cuda")
    X32 = X.float()
    L = oz.oz2_prepare_d(0, 0, 300, 200, X, 300, 14)
    R = oz.oz2_prepare_d(1, 0, 300, 200, X, 300, 14)
    C = torch.empty((300, 300), dtype=torch.float64, device="cuda")
    bad = [(R, R), (L, L), (L, oz.oz2_prepare_d(1, 0, 300, 100, X, 300, 14)),
           (L, oz.oz2_prepare_d(1, 0, 300, 200, X, 300, 15)), (L, oz.oz2_prepare_s(1, 0, 300, 200, X32, 300, 14))]
    for l, r in bad:
        with pytest.raises(oz.OZ2Error) as e:
            oz.oz2_dgemm_prepared(l, r, 1.0, 0.0, C, 300)
        assert e.value.status == 1
    with pytest.raises(oz.OZ2Error):
        oz.oz2_dgemm_prepared(L, R, 1.0, 0.0, C, 299)      # ldc < n
    with pytest.raises(oz.OZ2Error):
        oz.oz2_sgemm_prepared(L, R, 1.0, 0.0, C.float(), 300)
    oz.oz2_dgemm_prepared(L, R, 1.0, 0.0, C, 300)
    torch.cuda.synchronize()
    assert bool((C == 0).all())
    L.free(); L.free()                                     # idempotent


def test_prepared_operands_at_4096_with_panels(oz, oracle):
    """A 4096^3 product of prepared operands, whole and cut into 4 panels, against sampled
    oracle rows."""
    import torch
    m = n = k = 4096
    N = 15
    A, B = S.gemm_inputs(m, n, k, 0.5, seed=0)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    L = oz.oz2_prepare_d(0, 0, m, k, dA, k, N)
    R = oz.oz2_prepare_d(1, 0, n, k, dB, n, N)
    C1 = torch.empty((m, n), dtype=torch.float64, device="cuda")
    oz.oz2_dgemm_prepared(L, R, 1.0, 0.0, C1, n)
    assert oz.oz2_last_panels() == (4096, 4096, 1)
    assert torch.equal(C1, oz.matmul(dA, dB, N))
    try:
        oz.oz2_set_workspace_limit(N * 2048 * 2048 + 4096)
        oz.oz2_release()
        C2 = torch.empty_like(C1)
        oz.oz2_dgemm_prepared(L, R, 1.0, 0.0, C2, n)
        assert oz.oz2_last_panels() == (2048, 2048, 4)
        assert torch.equal(C1, C2)
    finally:
        oz.oz2_set_workspace_limit(0)
        oz.oz2_release()
    prep = oracle.prepare(A, B, N, True, False)
    rows = np.array([0, 1777, 4095])
    fin = oracle.finish_rows(prep, rows)
    assert np.array_equal(C1[torch.from_numpy(rows).cuda()].cpu().numpy(), fin["C"])
    L.free(); R.free()


def test_config_8192_transposed_and_panelled_sampled(oz, oracle):
    """Benchmark-class size: op(A) = A^T, op(B) = B^T, the product cut into 4 panels; shifts and
    residues compared in full, U_s of the last panel and C on sampled rows and entries."""
    import torch
    from paper_2508_03984_amd import binding as b
    m = n = k = 8192
    N = 16
    A, B = S.gemm_inputs(m, n, k, 1.0, seed=0)
    dAt = torch.from_numpy(A).cuda().t().contiguous()
    dBt = torch.from_numpy(B).cuda().t().contiguous()
    dC = torch.empty((m, n), dtype=torch.float64, device="cuda")
    least = oz.oz2_workspace_min_bytes(m, n, k, N)
    try:
        oz.oz2_set_workspace_limit(least - N * 256 * 256 + N * 4096 * 4096)
        oz.oz2_release()
        oz.oz2_dgemm_op(1, 1, 0, m, n, k, 1.0, dAt, m, dBt, k, 0.0, dC, n, N)
        torch.cuda.synchronize()
        assert oz.oz2_last_panels() == (4096, 4096, 4)
        prep = oracle.prepare(A, B, N, True, False)
        assert np.array_equal(oz.stage_tensor(b.OZ2_STAGE_SHIFT_A).cpu().numpy(), prep["tA"])
        assert np.array_equal(oz.stage_tensor(b.OZ2_STAGE_SHIFT_B).cpu().numpy(), prep["tB"])
        for stage, key, rows_ in ((b.OZ2_STAGE_RES_A, "Ares", m), (b.OZ2_STAGE_RES_B, "Bres", n)):
            r = oz.unblock_slices(oz.stage_tensor(stage, copy=False))
            for s in range(N):
                assert torch.equal(r[s, :rows_, :k], torch.from_numpy(prep[key][s]).cuda()), (key, s)
            del r
    finally:
        oz.oz2_set_workspace_limit(0)
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([[0, 4095, 4096, m - 1], rng.integers(0, m, 3)]))
    fin = oracle.finish_rows(prep, rows)
    assert np.array_equal(dC[torch.from_numpy(rows).cuda()].cpu().numpy(), fin["C"])
    ii = rng.integers(0, m, 800); jj = rng.integers(0, n, 800)
    ent = oracle.finish_entries(prep, ii, jj)
    assert np.array_equal(dC[torch.from_numpy(ii).cuda(), torch.from_numpy(jj).cuda()].cpu().numpy(), ent["C"])
    oz.oz2_release()


# ------------------------------------------------------------------ HIP graph capture
@pytest.mark.parametrize("accurate", [False, True])
def test_call_can_be_captured_into_a_hip_graph(oz, oracle, accurate):
    """A call allocates nothing once its workspace exists and clears its scratch with fill
    kernels, so it can be recorded into a HIP graph; every replay, with new contents in the
    same buffers and eager work in between, must equal the eager result."""
    import torch
    m, n, k, N = 300, 520, 700, 15
    A, B = S.gemm_inputs(m, n, k, 1.0, seed=90)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    dC = torch.zeros((m, n), dtype=torch.float64, device="cuda")
    oz.matmul(dA, dB, N, out=dC, accurate=accurate)           # allocates the workspace, eagerly
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):                                 # torch's current stream is the capture stream
        oz.matmul(dA, dB, N, out=dC, accurate=accurate)
    for rep in range(4):
        A2, B2 = S.gemm_inputs(m, n, k, 0.5 + 0.5 * rep, seed=91 + 2 * rep)
        if rep == 2:
            A2[7, :] = 0.0; B2[:, 11] = 0.0
        dA.copy_(torch.from_numpy(A2).cuda()); dB.copy_(torch.from_numpy(B2).cuda())
        dC.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        got = dC.clone()
        eager = oz.matmul(dA, dB, N, accurate=accurate)       # the program's own eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(got, eager), rep
        assert np.array_equal(got.cpu().numpy(), oracle.gemm(A2, B2, N, accurate=accurate)["C"]), rep
    del g


def test_prepared_transposed_operands_with_k_beyond_2_pow_17(oz, oracle):
    """Everything at once on a small C: A stored transposed, two K ranges folded modulo p_s,
    prepared operands, two panels."""
    import torch
    m, n, k, N = 40, 300, 2 ** 17 + 700, 13
    A, B = S.gemm_inputs(m, n, k, 0.5, seed=95)
    dAt = torch.from_numpy(np.ascontiguousarray(A.T)).cuda()
    dB = torch.from_numpy(B).cuda()
    want = oracle.gemm(A, B, N)["C"]
    L = oz.oz2_prepare_d(0, 1, m, k, dAt, m, N)
    R = oz.oz2_prepare_d(1, 0, n, k, dB, n, N)
    dC = torch.empty((m, n), dtype=torch.float64, device="cuda")
    try:
        oz.oz2_set_workspace_limit(N * 256 * 256)
        oz.oz2_release()
        oz.oz2_dgemm_prepared(L, R, 1.0, 0.0, dC, n)
        assert oz.oz2_last_panels() == (256, 256, 2)
        assert np.array_equal(dC.cpu().numpy(), want)
    finally:
        oz.oz2_set_workspace_limit(0)
        oz.oz2_release()
    assert np.array_equal(oz.matmul(dAt.t(), dB, N).cpu().numpy(), want)
    L.free(); R.free()


def test_random_shapes_modes_and_operand_forms_against_the_oracle(oz, oracle):
    """Seeded sweep over small random problems: shape, number of moduli, exponent spread, FP64 /
    FP32, fast / accurate mode, transpositions, alpha / beta, leading dimensions and an
    occasional workspace limit; integer stages bit-exact, C within the tolerance."""
    import torch
    rng = np.random.default_rng(2024)
    for case in range(120):
        is_double = bool(rng.integers(0, 2))
        dtype = np.float64 if is_double else np.float32
        m, n = int(rng.integers(1, 600)), int(rng.integers(1, 600))
        k = int(rng.choice([1, 7, 64, 129, 500, 1100, 2300]))
        N = int(rng.integers(2, 21))
        phi = float(rng.choice([0.5, 1.0, 2.0, 4.0]))
        accurate = bool(rng.integers(0, 2))
        opA, opB = int(rng.integers(0, 2)), int(rng.integers(0, 2))
        alpha, beta = (1.0, 0.0) if rng.integers(0, 2) else (float(rng.normal()), float(rng.normal()))
        if not is_double:                                  # oz2_sgemm_op takes alpha and beta as floats
            alpha, beta = float(np.float32(alpha)), float(np.float32(beta))
        A, B = S.gemm_inputs(m, n, k, phi, seed=1000 + 2 * case, dtype=dtype)
        if rng.integers(0, 4) == 0:
            A[int(rng.integers(0, m)), :] = 0.0
            B[:, int(rng.integers(0, n))] = 0.0
        Cin = S.matrix(m, n, 0.5, seed=3000 + case, dtype=dtype) if beta != 0.0 else None
        ref = oracle.gemm(A, B, N, alpha, beta, Cin, is_double=is_double, accurate=accurate)
        limited = bool(rng.integers(0, 3) == 0) and max(m, n) > 256
        try:
            if limited:
                oz.oz2_set_workspace_limit(oz.oz2_workspace_min_bytes(m, n, k, N, is_double))
                oz.oz2_release()
            got = run_op(oz, A, B, N, opA, opB, accurate, alpha, beta, Cin,
                         lda_extra=int(rng.integers(0, 9)), ldb_extra=int(rng.integers(0, 9)),
                         small_conversion=bool(case % 2)) \
                if not limited else None
            if limited:
                dt = torch.float64 if is_double else torch.float32
                dA, lda = stored(A, opA, 1, dt)
                dB, ldb = stored(B, opB, 2, dt)
                dC = torch.from_numpy(Cin).cuda() if Cin is not None else torch.empty((m, n), dtype=dt, device="cuda")
                fn = oz.oz2_dgemm_op if is_double else oz.oz2_sgemm_op
                fn(opA, opB, accurate, m, n, k, alpha, dA, lda, dB, ldb, beta, dC, n, N)
                assert oz.oz2_last_panels()[2] > 1
                c, r = dC.cpu().numpy().astype(np.float64), ref["C"].astype(np.float64)
                rel = np.max(np.abs(c - r) / np.where(r == 0, 1.0, np.abs(r)))
                assert rel <= (TOL64 if is_double else TOL32), (case, rel)
            else:
                check(got, ref, is_double)
        except AssertionError as e:
            raise AssertionError(f"case {case}: m={m} n={n} k={k} N={N} phi={phi} {dtype.__name__} "
                                 f"accurate={accurate} op=({opA},{opB}) alpha={alpha} beta={beta} "
                                 f"limited={limited}: {e}")
        finally:
            if limited:
                oz.oz2_set_workspace_limit(0)
                oz.oz2_release()


# ------------------------------------------------------------------ small problems
@pytest.mark.parametrize("accurate", [False, True])
@pytest.mark.parametrize("m,n,k,N,dtype,opA,opB", [
    (2048, 2048, 2048, 14, np.float64, 0, 0),      # the largest cube the fused launches take
    (1500, 2500, 2000, 16, np.float64, 1, 1),      # A by columns, B by rows
    (8192, 3, 1000, 13, np.float64, 0, 0),         # many short rows, three columns
    (5, 8192, 1020, 20, np.float64, 1, 0),         # both factors by columns
    (1024, 1000, 4096, 8, np.float32, 0, 0),       # the longest columns; strips of 16
    (1000, 1024, 4095, 9, np.float32, 0, 1),       # both factors by rows
])
def test_small_conversion_equals_the_general_kernels(oz, m, n, k, N, dtype, opA, opB, accurate):
    """Up to (m + n) k = 2 x 2048^2 the shifts and residues of both factors come from two fused
    launches; every stage and C must equal what the general kernels give, bit for bit (those
    are checked against the oracle at these sizes by the sampled tests)."""
    import torch
    from paper_2508_03984_amd import binding as b
    A, B = S.gemm_inputs(m, n, k, 2.0, seed=77 + N, dtype=dtype)
    A[m // 2, :] = 0.0
    B[:, n // 3] = 0.0
    is_double = dtype == np.float64
    dt = torch.float64 if is_double else torch.float32
    dA, lda = stored(A, opA, 2, dt)
    dB, ldb = stored(B, opB, 6, dt)
    fn = oz.oz2_dgemm_op if is_double else oz.oz2_sgemm_op
    got = {}
    try:
        for small in (True, False):
            oz.oz2_set_small_conversion(small)
            dC = torch.full((m, n), float("nan"), dtype=dt, device="cuda")
            fn(opA, opB, accurate, m, n, k, 1.0, dA, lda, dB, ldb, 0.0, dC, n, N)
            torch.cuda.synchronize()
            got[small] = [dC] + [oz.stage_tensor(st) for st in (b.OZ2_STAGE_SHIFT_A, b.OZ2_STAGE_SHIFT_B,
                                                                 b.OZ2_STAGE_RES_A, b.OZ2_STAGE_RES_B)]
    finally:
        oz.oz2_set_small_conversion(True)
    for x, y, name in zip(got[True], got[False], ("C", "tA", "tB", "residues of A", "residues of B")):
        assert torch.equal(x, y), name
    assert int(got[True][1][m // 2]) == 0 and int(got[True][2][n // 3]) == 0     # zero vectors: shift 0
    assert bool(torch.isfinite(got[True][0]).all())


# ------------------------------------------------------------------ overlapped form
@pytest.mark.parametrize("opA,opB,accurate", [(0, 0, False), (1, 1, False), (1, 0, True)])
def test_overlapped_form_equals_the_single_stream_form(oz, oracle, opA, opB, accurate):
    """k >= 8192 and a padded C of 8448 x 8704 (3 x 3 panels with ragged last ones): the overlapped
    form converts the blocks of A and B on a second stream while the GEMMs of earlier panels
    run; it must equal the single-stream form bit for bit, call after call, and the oracle."""
    import torch
    from paper_2508_03984_amd import binding as b
    m, n, k, N = 8300, 8500, 8200, 13
    A, B = S.gemm_inputs(m, n, k, 1.0, seed=110)
    Cin = S.matrix(m, n, 0.5, seed=111)
    dA, lda = stored(A, opA, 1, torch.float64)
    dB, ldb = stored(B, opB, 3, torch.float64)

    def run():
        dC = torch.from_numpy(Cin).cuda()
        oz.oz2_dgemm_op(opA, opB, accurate, m, n, k, 0.5, dA, lda, dB, ldb, -1.25, dC, n, N)
        return dC

    oz.oz2_set_overlap(False)
    try:
        want = run()
        assert oz.oz2_last_panels()[2] == 1
    finally:
        oz.oz2_set_overlap(True)
    for rep in range(3):
        got = run()
        assert oz.oz2_last_panels() == (4096, 4096, 9)
        assert torch.equal(got, want), rep
    with pytest.raises(oz.OZ2Error):                       # the products of all of C are not kept
        oz.oz2_stage_ptr(b.OZ2_STAGE_U)
    prep = oracle.prepare(A, B, N, True, accurate)
    assert np.array_equal(oz.stage_tensor(b.OZ2_STAGE_SHIFT_A).cpu().numpy(), prep["tA"])
    assert np.array_equal(oz.stage_tensor(b.OZ2_STAGE_SHIFT_B).cpu().numpy(), prep["tB"])
    ra = oz.unblock_slices(oz.stage_tensor(b.OZ2_STAGE_RES_A, copy=False))
    rb = oz.unblock_slices(oz.stage_tensor(b.OZ2_STAGE_RES_B, copy=False))
    for s_ in range(N):                                    # residues written block by block, padding zero
        assert torch.equal(ra[s_, :m, :k], torch.from_numpy(prep["Ares"][s_]).cuda())
        assert torch.equal(rb[s_, :n, :k], torch.from_numpy(prep["Bres"][s_]).cuda())
        assert bool((ra[s_, m:, :] == 0).all() and (ra[s_, :, k:] == 0).all())
        assert bool((rb[s_, n:, :] == 0).all() and (rb[s_, :, k:] == 0).all())
    del ra, rb
    rows = np.array([0, 4095, 4096, 8191, 8192, m - 1])
    fin = oracle.finish_rows(prep, rows, 0.5, -1.25, np.ascontiguousarray(Cin[rows]))
    assert np.array_equal(want[torch.from_numpy(rows).cuda()].cpu().numpy(), fin["C"])
    oz.oz2_release()


def test_overlapped_form_with_k_ranges_fp32_and_a_workspace_limit(oz, oracle):
    """Two K ranges per panel and FP32; a workspace limit cuts a C of 4352 x 4608 into nine
    panels of 2048 x 2048, which makes the call an overlapped one."""
    import torch
    m, n, k, N = 4200, 4400, 2 ** 17 + 200, 5
    A, B = S.gemm_inputs(m, n, k, 0.5, seed=112, dtype=np.float32)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    oz.oz2_set_overlap(False)
    try:
        want = oz.matmul(dA, dB, N)
        assert oz.oz2_last_panels() == (4352, 4608, 1)
        assert oz.oz2_last_gemm_launches() == 4            # 4096 + 256 rows, two K ranges each
    finally:
        oz.oz2_set_overlap(True)
    got = oz.matmul(dA, dB, N)                             # four panels, and k is long enough to overlap
    assert oz.oz2_last_panels() == (4096, 4096, 4) and torch.equal(got, want)
    least = oz.oz2_workspace_min_bytes(m, n, k, N, False)
    try:
        oz.oz2_set_workspace_limit(least - 5 * 256 * 256 + 5 * 2048 * 2048)
        oz.oz2_release()
        got = oz.matmul(dA, dB, N)
        assert oz.oz2_last_panels() == (2048, 2048, 9) and torch.equal(got, want)
        oz.oz2_set_overlap(False)
        got = oz.matmul(dA, dB, N)
        assert oz.oz2_last_panels() == (2048, 2048, 9) and torch.equal(got, want)
    finally:
        oz.oz2_set_overlap(True)
        oz.oz2_set_workspace_limit(0)
        oz.oz2_release()
    rows = np.array([0, 4199])
    ref = oracle.gemm(A[rows], B, N, is_double=False)["C"]
    assert np.array_equal(want[torch.from_numpy(rows).cuda()].cpu().numpy(), ref)


def test_overlapped_call_in_a_hip_graph(oz):
    """The second stream forks from and joins the caller's stream, so the overlapped call can be
    captured; replays with new inputs equal the eager results."""
    import torch
    m, n, k, N = 2100, 2300, 8192, 12
    A, B = S.gemm_inputs(m, n, k, 0.5, seed=113)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    dC = torch.zeros((m, n), dtype=torch.float64, device="cuda")
    least = oz.oz2_workspace_min_bytes(m, n, k, N)
    try:
        oz.oz2_set_workspace_limit(least - N * 256 * 256 + N * 512 * 512)
        oz.oz2_release()
        oz.matmul(dA, dB, N, out=dC)                       # workspace, second stream and events exist now
        assert oz.oz2_last_panels() == (512, 512, 25)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            oz.matmul(dA, dB, N, out=dC)
        for rep in range(3):
            A2, B2 = S.gemm_inputs(m, n, k, 1.0, seed=114 + 2 * rep)
            dA.copy_(torch.from_numpy(A2).cuda()); dB.copy_(torch.from_numpy(B2).cuda())
            dC.fill_(float("nan"))
            g.replay()
            torch.cuda.synchronize()
            got = dC.clone()
            assert torch.equal(got, oz.matmul(dA, dB, N)), rep
        del g
    finally:
        oz.oz2_set_workspace_limit(0)
        oz.oz2_release()


def test_overlapped_form_with_int32_products(oz):
    """The diagnostic pipeline (INT32 sums kept, reduced in the accumulation) in the overlapped
    form: same result as the default uint8 pipeline, bit for bit."""
    import torch
    m, n, k, N = 2100, 2300, 8192, 12
    A, B = S.gemm_inputs(m, n, k, 2.0, seed=117)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    try:
        for int32 in (False, True):
            oz.oz2_set_int32_products(int32)
            least = oz.oz2_workspace_min_bytes(m, n, k, N)
            per = 4 * N if int32 else N
            oz.oz2_set_workspace_limit(least - per * 256 * 256 + per * 512 * 512)
            oz.oz2_release()
            got = oz.matmul(dA, dB, N)
            assert oz.oz2_last_panels() == (512, 512, 25)
            if int32:
                assert torch.equal(got, want)
            want = got
    finally:
        oz.oz2_set_int32_products(False)
        oz.oz2_set_workspace_limit(0)
        oz.oz2_release()


def test_overlapped_form_in_a_caller_owned_workspace(oz):
    """A caller-owned buffer sized for panels of 512 x 512: the overlapped form runs in it,
    allocates no workspace of its own, and gives the result of the library-owned workspace."""
    import torch
    m, n, k, N = 2100, 2300, 8192, 12
    A, B = S.gemm_inputs(m, n, k, 0.5, seed=118)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    want = oz.matmul(dA, dB, N)
    oz.oz2_release()
    least = oz.oz2_workspace_min_bytes(m, n, k, N)
    buf = torch.empty(least - N * 256 * 256 + N * 512 * 512, dtype=torch.uint8, device="cuda")
    oz.oz2_set_workspace(buf)
    try:
        got = torch.empty_like(want)
        oz.matmul(dA, dB, N, out=got)                          # creates the second stream and its events
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        got.zero_()
        oz.matmul(dA, dB, N, out=got)
        torch.cuda.synchronize()
        assert oz.oz2_last_panels() == (512, 512, 25)
        # no workspace of the library's own (it would be some 250 MB; the runtime's own pools may grow a little)
        assert free_before - torch.cuda.mem_get_info()[0] < 32 * 2 ** 20
        assert torch.equal(got, want)
    finally:
        oz.oz2_set_workspace(None)
        oz.oz2_release()


def test_stage_times_after_an_overlapped_and_then_a_prepared_call(oz):
    """The stage times belong to the last call, whatever form the call before it had."""
    import torch
    m, n, k, N = 2100, 2300, 8192, 12
    A, B = S.gemm_inputs(m, n, k, 0.5, seed=120)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    dC = torch.empty((m, n), dtype=torch.float64, device="cuda")
    least = oz.oz2_workspace_min_bytes(m, n, k, N)
    oz.oz2_set_profiling(True)
    try:
        oz.oz2_set_workspace_limit(least - N * 256 * 256 + N * 512 * 512)
        oz.oz2_release()
        oz.matmul(dA, dB, N, out=dC)                       # overlapped: 25 panels
        assert oz.oz2_last_panels()[2] == 25
        t = oz.oz2_last_stage_times_ms()
        assert all(x >= 0.0 for x in t) and 0.0 < sum(t) < 1000.0, t
        oz.oz2_set_workspace_limit(0)
        L = oz.oz2_prepare_d(0, 0, m, k, dA, k, N)
        R = oz.oz2_prepare_d(1, 0, n, k, dB, n, N)
        oz.oz2_dgemm_prepared(L, R, 1.0, 0.0, dC, n)
        t = oz.oz2_last_stage_times_ms()
        assert all(x >= 0.0 for x in t) and 0.0 < sum(t) < 1000.0, t
        oz.matmul(dA[:300], dB, N)                         # a small plain call
        t = oz.oz2_last_stage_times_ms()
        assert all(x >= 0.0 for x in t) and 0.0 < sum(t) < 1000.0, t
        L.free(); R.free()
    finally:
        oz.oz2_set_profiling(False)
        oz.oz2_set_workspace_limit(0)
        oz.oz2_release()
