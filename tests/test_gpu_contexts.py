"""GPU tests of contexts (oz2_create / oz2_ctx_*): products of different contexts run
concurrently on different streams and from different host threads, each with a workspace, options
and diagnostics of its own, and every one of them equals the CPU oracle."""
import threading

import numpy as np
import pytest

import synth_inputs as S

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def oz():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2508_03984_amd as oz
    oz.load()
    yield oz
    oz.oz2_release()


def stages_equal_oracle(oz, ctx, ref, m, n, k):
    from paper_2508_03984_amd import binding as b
    assert np.array_equal(oz.stage_tensor(b.OZ2_STAGE_SHIFT_A, ctx=ctx).cpu().numpy(), ref["tA"])
    assert np.array_equal(oz.stage_tensor(b.OZ2_STAGE_SHIFT_B, ctx=ctx).cpu().numpy(), ref["tB"])
    ra = oz.unblock_slices(oz.stage_tensor(b.OZ2_STAGE_RES_A, ctx=ctx))[:, :m, :k].cpu().numpy()
    rb = oz.unblock_slices(oz.stage_tensor(b.OZ2_STAGE_RES_B, ctx=ctx))[:, :n, :k].cpu().numpy()
    assert np.array_equal(ra, ref["Ares"]) and np.array_equal(rb, ref["Bres"])
    assert np.array_equal(oz.stage_tensor(b.OZ2_STAGE_U, ctx=ctx)[:, :m, :n].cpu().numpy(), ref["U"])


def test_two_contexts_on_two_streams_concurrently(oz, oracle):
    """Two different products (FP64 with 15 moduli, FP32 with 8) issued alternately on two streams
    without any synchronisation between them: each context has its own workspace, so neither
    disturbs the other; results and every integer stage equal the oracle's bit for bit."""
    import torch
    A1, B1 = S.gemm_inputs(1900, 1700, 1500, 1.0, seed=200)
    A2, B2 = S.gemm_inputs(1300, 2200, 1100, 0.5, seed=202, dtype=np.float32)
    ref1 = oracle.gemm(A1, B1, 15)
    ref2 = oracle.gemm(A2, B2, 8, is_double=False)
    dA1, dB1 = torch.from_numpy(A1).cuda(), torch.from_numpy(B1).cuda()
    dA2, dB2 = torch.from_numpy(A2).cuda(), torch.from_numpy(B2).cuda()
    c1, c2 = oz.Context(), oz.Context()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    C1 = torch.empty((1900, 1700), dtype=torch.float64, device="cuda")
    C2 = torch.empty((1300, 2200), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    for rep in range(6):
        C1.fill_(float("nan")); C2.fill_(float("nan"))
        torch.cuda.synchronize()
        oz.matmul(dA1, dB1, 15, out=C1, stream=s1, ctx=c1)
        oz.matmul(dA2, dB2, 8, out=C2, stream=s2, ctx=c2)
        oz.matmul(dA1, dB1, 15, out=C1, stream=s1, ctx=c1)       # back to back on the same stream: ordered
        torch.cuda.synchronize()
        assert np.array_equal(C1.cpu().numpy(), ref1["C"]), rep
        assert np.array_equal(C2.cpu().numpy(), ref2["C"]), rep
    stages_equal_oracle(oz, c1, ref1, 1900, 1700, 1500)
    stages_equal_oracle(oz, c2, ref2, 1300, 2200, 1100)
    assert oz.oz2_ctx_last_panels(c1) == (2048, 1792, 1) and oz.oz2_ctx_last_panels(c2) == (1536, 2304, 1)
    c1.destroy(); c2.destroy()


def test_contexts_from_two_host_threads(oz, oracle):
    """Two host threads, each with a context and a stream of its own, issue products at the same
    time (accurate mode in one of them); every result equals the oracle's."""
    import torch
    A1, B1 = S.gemm_inputs(700, 900, 2100, 2.0, seed=210)
    A2, B2 = S.gemm_inputs(1100, 600, 800, 0.5, seed=212)
    ref = [oracle.gemm(A1, B1, 16, accurate=True)["C"], oracle.gemm(A2, B2, 13)["C"]]
    dev = [(torch.from_numpy(A1).cuda(), torch.from_numpy(B1).cuda(), 16, True),
           (torch.from_numpy(A2).cuda(), torch.from_numpy(B2).cuda(), 13, False)]
    ctxs = [oz.Context(), oz.Context()]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    bad, errors = [0, 0], []
    torch.cuda.synchronize()

    def work(i):
        try:
            torch.cuda.set_device(0)
            dA, dB, N, accurate = dev[i]
            want = torch.from_numpy(ref[i]).cuda()
            for _ in range(12):
                got = oz.matmul(dA, dB, N, accurate=accurate, stream=streams[i], ctx=ctxs[i])
                streams[i].synchronize()
                bad[i] += int(not torch.equal(got, want))
        except Exception as ex:                              # surfaced in the main thread below
            errors.append(ex)

    threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    assert bad == [0, 0]
    for c in ctxs:
        c.destroy()


def test_options_and_workspaces_belong_to_their_context(oz, oracle):
    import torch
    from paper_2508_03984_amd import binding as b
    A, B = S.gemm_inputs(300, 280, 500, 0.5, seed=220)
    ref = oracle.gemm(A, B, 14)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    c = oz.Context()
    oz.oz2_ctx_set_option(c, b.OZ2_OPT_INT32_PRODUCTS, True)
    assert oz.oz2_ctx_workspace_bytes(c, 300, 280, 500, 14) > oz.oz2_workspace_bytes(300, 280, 500, 14)
    got_c = oz.matmul(dA, dB, 14, ctx=c)
    got_default = oz.matmul(dA, dB, 14)
    torch.cuda.synchronize()
    assert np.array_equal(got_c.cpu().numpy(), ref["C"]) and np.array_equal(got_default.cpu().numpy(), ref["C"])
    assert np.array_equal(oz.stage_tensor(b.OZ2_STAGE_PROD, ctx=c)[:, :300, :280].cpu().numpy(), ref["prod"])
    assert np.array_equal(oz.stage_tensor(b.OZ2_STAGE_U)[:, :300, :280].cpu().numpy(), ref["U"])
    with pytest.raises(oz.OZ2Error):
        oz.oz2_ctx_stage_ptr(c, b.OZ2_STAGE_U)               # this context keeps the INT32 form
    with pytest.raises(oz.OZ2Error):
        oz.oz2_stage_ptr(b.OZ2_STAGE_PROD)                   # the default context does not
    # a caller-owned workspace on the context, too small and then large enough
    need = oz.oz2_ctx_workspace_bytes(c, 300, 280, 500, 14)
    small = torch.empty(oz.oz2_ctx_workspace_min_bytes(c, 300, 280, 500, 14) - 256, dtype=torch.uint8, device="cuda")
    oz.oz2_ctx_set_workspace(c, small)
    with pytest.raises(oz.OZ2Error) as e:
        oz.matmul(dA, dB, 14, ctx=c)
    assert e.value.status == 3
    buf = torch.empty(need, dtype=torch.uint8, device="cuda")
    oz.oz2_ctx_set_workspace(c, buf)
    assert np.array_equal(oz.matmul(dA, dB, 14, ctx=c).cpu().numpy(), ref["C"])
    assert buf.data_ptr() <= oz.oz2_ctx_stage_ptr(c, b.OZ2_STAGE_SHIFT_A)[0] < buf.data_ptr() + need   # it works in that buffer
    oz.oz2_ctx_set_workspace(c, None)
    with pytest.raises(oz.OZ2Error):
        oz.oz2_ctx_set_option(c, 17, 1)
    oz.oz2_ctx_set_option(c, b.OZ2_OPT_PROFILING, True)
    oz.matmul(dA, dB, 14, ctx=c)
    t = oz.oz2_ctx_last_stage_times_ms(c)
    assert all(x >= 0.0 for x in t) and 0.0 < sum(t) < 100.0
    with pytest.raises(oz.OZ2Error):
        oz.oz2_last_stage_times_ms()                         # profiling is off in the default context
    c.destroy()


def test_destroy_frees_the_workspace(oz):
    import torch
    m = n = k = 4096
    dA = torch.ones((m, k), dtype=torch.float64, device="cuda")
    out = torch.empty((m, n), dtype=torch.float64, device="cuda")
    c = oz.Context()
    torch.cuda.synchronize()
    before = torch.cuda.mem_get_info()[0]
    oz.matmul(dA, dA, 16, out=out, ctx=c)
    torch.cuda.synchronize()
    held = before - torch.cuda.mem_get_info()[0]
    assert held >= oz.oz2_ctx_workspace_bytes(c, m, n, k, 16)
    c.destroy()
    assert before - torch.cuda.mem_get_info()[0] < held // 2
