"""xbar_fwd_static (workspace in the library's static per-GPU array, no allocation) against xbar_fwd:
same kernels, so the outputs must be bit-identical; two calls in a row, the second on a smaller input."""
import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def test_fwd_static_equals_fwd_twice():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2002_11151_amd import xbar as xb
    xb.lib()
    kw = workloads.config_kwargs("resnet50")
    cfg = xb.make_config(**kw)
    for M, K, N in ((300, 576, 130), (70, 147, 64)):          # second call: smaller input, ragged tiles
        g = workloads.Gemm("t", K, N, M, False, 1)
        W, X, _ = workloads.layer_tensors_np(g, seed=11 + M)
        w_max, xs = float(np.abs(W).max()), float(np.abs(X).max())
        Wd, Xd = torch.from_numpy(W).cuda(), torch.from_numpy(X).cuda()
        planes = xb.tile(cfg, Wd, w_max, 3)
        want = xb.fwd(cfg, planes, Xd, N, w_max, xs)
        got = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        before = torch.cuda.memory_allocated()
        xb.fwd_static(cfg, planes, Xd, N, w_max, xs, out=got)
        assert torch.cuda.memory_allocated() == before       # the binding allocates nothing either
        torch.cuda.synchronize()
        assert torch.equal(got, want), "static-scratch forward differs from xbar_fwd at M=%d" % M
    # a shape beyond the static array is refused, and nothing is enqueued
    big_M = 1 << 22
    assert xb.workspace_bytes(cfg, xb.OP_FWD, big_M, 576, 64) > (32 << 20)
    planes = xb.tile(cfg, torch.zeros((576, 64), device="cuda"), 1.0, 0)
    code = xb.lib().xbar_fwd_static(xb.C.byref(cfg), xb.C.c_void_p(planes.data_ptr()), xb.C.c_void_p(planes.data_ptr()),
                                    xb.C.c_void_p(planes.data_ptr()), big_M, 576, 64, 1.0, 1.0, None)
    assert code == -7 and "static" in xb.strerror(code)
