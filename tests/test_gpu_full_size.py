"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py
times (ResNet-50 layer GEMMs at batch 64 = the benchmarked workload; one layer each of the ResNet-20
and VGG-16 configurations): the HIP path runs the whole layer, the oracle recomputes sampled batch
rows (forward, backward) and a sampled block of weights (update) one by one."""
import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

LAYERS = [("resnet50", 64, "conv1_7x7"), ("resnet50", 64, "s1b0_1x1b"), ("resnet50", 64, "s4b0_3x3"),
          ("resnet20", 128, "s1b0_a"),        # 16 output columns: half-empty output patch, 4-bit cycles
          ("vgg16", 128, "conv1_2")]          # 6.4 M rows (M*K > 2^31), 256x256 tiles, device variation


@pytest.fixture(scope="module")
def xb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2002_11151_amd import xbar
    xbar.lib()
    return xbar


def rel_l2(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


@pytest.mark.parametrize("workload,batch,name", LAYERS)
def test_layer_full_size_sampled(xo, xb, workload, batch, name):
    gemms = {g.name: (i, g) for i, g in enumerate(workloads.GEMMS[workload](batch, merge=True))}
    idx, g = gemms[name]
    kw = workloads.config_kwargs(workload)
    kw["flags"] |= workloads.INPUT_SIGNED if g.signed_input else 0
    co, cg = xo.make_config(**kw), xb.make_config(**kw)
    W, X, dY = workloads.layer_tensors_torch(g, seed=idx, device="cuda")
    w_max = 2.0 * float(W.abs().max())
    xs, gs = float(X.abs().max()), float(dY.abs().max())
    planes = xb.tile(cg, W, w_max, 5)
    Y = xb.fwd(cg, planes, X, g.N, w_max, xs)
    dX = xb.bwd(cg, planes, dY, g.K, w_max, gs)
    W_new = W.clone()
    xb.update(cg, W_new, X, dY, w_max, 1.0 / w_max, 0.01, 5)
    torch.cuda.synchronize()

    rng = np.random.default_rng(idx)
    rows = np.sort(rng.choice(g.M, size=8, replace=False))
    rows[0], rows[-1] = 0, g.M - 1                       # first and last row of the ragged tail
    rt = torch.from_numpy(rows).cuda()
    Wh = W.cpu().numpy()
    U = xo.planes(co, Wh, w_max, 5)
    Yo = xo.rows_parallel(lambda u, x: xo.fwd_planes(co, u, x, w_max, xs), U, X[rt].cpu().numpy(), 8)
    dXo = xo.rows_parallel(lambda u, x: xo.bwd_planes(co, u, x, w_max, gs), U, dY[rt].cpu().numpy(), 8)
    assert rel_l2(Y[rt].cpu().numpy(), Yo) <= 1e-3
    assert rel_l2(dX[rt].cpu().numpy(), dXo) <= 1e-3
    # every element within one top-slice LSB of the oracle (a flipped code moves one output by at most that)
    q_adc = (1 << (kw["adc_bits"] - 1)) - 1
    top_shift = kw["weight_bits"] - kw["slice_bits"] + kw["input_bits"] - kw["stream_bits"]
    lsb_f = kw["adc_fs_fwd"] / q_adc * xs * w_max / (255.0 * ((1 << kw["weight_bits"]) - 1)) * 2 ** top_shift
    assert np.abs(Y[rt].cpu().numpy() - Yo).max() <= 1.01 * lsb_f

    k_idx = np.sort(rng.choice(g.K, size=min(6, g.K), replace=False))
    n_idx = np.sort(rng.choice(g.N, size=min(5, g.N), replace=False))
    kt, nt = torch.from_numpy(k_idx).cuda(), torch.from_numpy(n_idx).cuda()
    Wo = xo.update(co, Wh[np.ix_(k_idx, n_idx)], X[:, kt].cpu().numpy(), dY[:, nt].cpu().numpy(), w_max,
                   1.0 / w_max, 0.01, step=5, k_idx=k_idx, n_idx=n_idx, N_full=g.N)
    Wg = W_new[kt][:, nt].cpu().numpy()
    assert rel_l2(Wg - Wh[np.ix_(k_idx, n_idx)], Wo - Wh[np.ix_(k_idx, n_idx)]) <= 1e-3
