"""artopk_variance_static, the entry point for callers that cannot allocate: called through the
C ABI twice in a row (the second time on a smaller problem, so that the fixed scratch still holds
the first call's partial results) and compared with artopk_variance on the same inputs -- same
kernels, same launch shape, hence the same bits -- and with the oracle's two-pass variance."""

import ctypes as C

import numpy as np
import pytest

from oracle import artopk_oracle as orc

pytestmark = pytest.mark.gpu


def _call_static(lib, x, var, argmax, stream):
    table = (C.c_void_p * len(x))(*[int(t.data_ptr()) for t in x])
    return lib.artopk_variance_static(table, len(x), x[0].numel(), C.c_void_p(int(var.data_ptr())),
                                      C.c_void_p(int(argmax.data_ptr())), C.c_void_p(stream))


def test_variance_static_matches_variance_on_two_calls_in_a_row():
    import torch
    import paper_2312_02493_amd as pkg

    lib = pkg.load_library()
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    rng = np.random.default_rng(2312)
    # the second problem is smaller in both W and N: it uses fewer blocks and fewer workers' slots
    for w, n in ((6, 3_000_017), (3, 70_001)):
        host = [(rng.standard_normal(n) * (0.5 + 0.25 * r) + 0.1 * r).astype(np.float32) for r in range(w)]
        x = [torch.from_numpy(a).to(dev) for a in host]
        ref = np.array([orc.variance(a) for a in host])

        ctx = pkg.Context(w, n, 1)
        var_ctx = torch.full((w,), -1.0, dtype=torch.float64, device=dev)
        am_ctx = torch.full((1,), -1, dtype=torch.int32, device=dev)
        ctx.artopk_variance(x, var_ctx, am_ctx)
        ctx.status()

        var = torch.full((w,), -2.0, dtype=torch.float64, device=dev)
        am = torch.full((1,), -2, dtype=torch.int32, device=dev)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        rc = _call_static(lib, x, var, am, stream)
        assert rc == 0, lib.artopk_last_error(None).decode()
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before

        got, want = var.cpu().numpy(), var_ctx.cpu().numpy()
        assert np.array_equal(got.view(np.uint64), want.view(np.uint64)), (got, want)
        assert int(am.item()) == int(am_ctx.item()) == orc.leader_var(list(ref))
        np.testing.assert_allclose(got, ref, rtol=1e-5, atol=0.0)
        for t, h in zip(x, host):   # inputs untouched
            assert np.array_equal(t.cpu().numpy().view(np.uint32), h.view(np.uint32))
        del ctx


def test_variance_static_rejects_what_its_scratch_cannot_hold():
    import torch
    import paper_2312_02493_amd as pkg

    lib = pkg.load_library()
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    x = [torch.zeros(64, device=dev) for _ in range(65)]
    var = torch.zeros(65, dtype=torch.float64, device=dev)
    am = torch.zeros(1, dtype=torch.int32, device=dev)
    assert _call_static(lib, x, var, am, stream) == -1          # 65 workers: more than the fixed scratch holds
    assert b"outside" in lib.artopk_last_error(None)
    table = (C.c_void_p * 1)(int(x[0].data_ptr()))
    assert lib.artopk_variance_static(table, 1, 1 << 31, C.c_void_p(int(var.data_ptr())), None, C.c_void_p(stream)) == -1
    assert lib.artopk_variance_static(table, 1, 0, C.c_void_p(int(var.data_ptr())), None, C.c_void_p(stream)) == -1
    assert lib.artopk_variance_static(table, 1, 64, None, None, C.c_void_p(stream)) == -1
    assert lib.artopk_variance_static(table, 1, 64, C.c_void_p(int(x[0].data_ptr())), None, C.c_void_p(stream)) == -1  # var_out over x
    # a call the scratch does hold still works afterwards
    assert _call_static(lib, x[:64], var, am, stream) == 0
    torch.cuda.synchronize()
    assert not var[:64].cpu().numpy().any()
