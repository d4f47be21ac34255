"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py
times (ResNet-50 layer GEMMs at batch 64 = the benchmarked workload; one layer each of the ResNet-20
and VGG-16 configurations): the HIP path runs the whole layer, the oracle recomputes sampled batch
rows (forward, backward) and a sampled block of weights (update) one by one."""
import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

# every one of the 24 distinct layer shapes of the benchmarked ResNet-50 workload -- among them the classifier (64
# batch rows, 2048 x 1000 weights), 64 x 64 weights (one half-filled crossbar, 200704 rows), the 1 x 1 projection
# shortcuts, and backward passes with more virtual tiles per chunk than 32-bit sums hold -- and one layer each of
# the ResNet-20 (16 output columns: half-empty output patch, 4-bit cycles) and VGG-16 configurations (6.4 M rows,
# M*K > 2^31, 256 x 256 tiles, device variation)
LAYERS = [("resnet50", 64, g.name) for g in workloads.resnet50_gemms(64, merge=True)] + \
         [("resnet20", 128, "s1b0_a"), ("vgg16", 128, "conv1_2")]


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


@pytest.mark.parametrize("variant", ["per_array", "offset", "offset+per_array", "adc12"])
def test_converter_and_streaming_variants_full_size_sampled(xo, xb, variant):
    """One ResNet-50 layer (4608 x 512, 3136 rows) in the launch configuration of `bench.py --adc-per-array`
    / `--offset-inputs` / `--adc-bits 12` (sums beyond 32 bits): sampled batch rows against the oracle."""
    gemms = {g.name: (i, g) for i, g in enumerate(workloads.resnet50_gemms(64, merge=True))}
    idx, g = gemms["s4b0_3x3"]
    kw = workloads.config_kwargs("resnet50")
    if "per_array" in variant:
        kw["flags"] |= workloads.ADC_PER_ARRAY
    if variant == "adc12":
        kw["adc_bits"] = 12
    if "offset" in variant:
        kw["flags"] |= workloads.INPUT_OFFSET
        kw["adc_fs_fwd"] *= 4.0
        kw["adc_fs_bwd"] *= 4.0
    co, cg = xo.make_config(**kw), xb.make_config(**kw)
    W, X, dY = workloads.layer_tensors_torch(g, seed=idx, device="cuda")
    w_max = 2.0 * float(W.abs().max())
    xs, gs = float(X.abs().max()), float(dY.abs().max())
    planes = xb.tile(cg, W, w_max, 5)
    Y = xb.fwd(cg, planes, X, g.N, w_max, xs)
    dX = xb.bwd(cg, planes, dY, g.K, w_max, gs)
    torch.cuda.synchronize()
    rng = np.random.default_rng(idx)
    rows = np.sort(rng.choice(g.M, size=8, replace=False))
    rows[0], rows[-1] = 0, g.M - 1
    rt = torch.from_numpy(rows).cuda()
    Wh = W.cpu().numpy()
    U = xo.planes(co, Wh, w_max, 5)
    col, row = xo.weight_sums(co, Wh, w_max)
    Yo = xo.rows_parallel(lambda u, x: xo.fwd_planes(co, u, x, w_max, xs, wsum=col), U, X[rt].cpu().numpy(), 8)
    dXo = xo.rows_parallel(lambda u, x: xo.bwd_planes(co, u, x, w_max, gs, wsum=row), U, dY[rt].cpu().numpy(), 8)
    # the forward input of this layer is unsigned (two-phase / offset coding only concern the backward pass)
    assert rel_l2(Y[rt].cpu().numpy(), Yo) <= 1e-3
    q_adc = (1 << kw["adc_bits"]) - 1 if "per_array" in variant else (1 << (kw["adc_bits"] - 1)) - 1
    top_shift = kw["weight_bits"] - kw["slice_bits"] + kw["input_bits"] - kw["stream_bits"]
    lsb_b = kw["adc_fs_bwd"] / q_adc * gs * w_max / (255.0 * ((1 << kw["weight_bits"]) - 1)) * 2 ** top_shift
    lsb_b *= 2.0 if "offset" in variant else 1.0
    got = dX[rt].cpu().numpy()
    assert np.abs(got - dXo).max() <= 1.01 * lsb_b          # no element is off by more than one top-slice code
    if "offset" in variant:
        # Offset coding: the output is an exact linear function of the codes, so it can differ from the oracle's
        # only by the weights of differing codes.  Under the code bar (at most 1e-4 of the conversions, one LSB
        # each) at most 1e-4 x (conversions per output) of the outputs are touched, each by at most one
        # top-slice code: that is the L2 bound asserted here (no codes are reported at this size).
        conversions = -(-g.N // kw["xbar_cols"]) * (kw["weight_bits"] // kw["slice_bits"]) * (kw["input_bits"] // kw["stream_bits"])
        touched = min(1.0, 1e-4 * conversions) * got.size
        assert np.linalg.norm(got - dXo) <= lsb_b * np.sqrt(touched)
        assert (got != dXo).mean() <= 1e-4 * conversions
    else:
        assert rel_l2(got, dXo) <= 1e-3


@pytest.mark.parametrize("name,ni", [("s4b0_3x3", "nl+noise"), ("s3b0_1x1b", "noise")])
def test_pulsed_update_full_size_sampled(xo, xb, name, ni):
    """Pulse-level update of whole ResNet-50 layers in the configuration `bench.py --pulsed-update` times
    (4608 x 512 devices: 4 x 4 per thread; 256 x 1024: marking pass and walk): sampled devices against the oracle."""
    gemms = {g.name: (i, g) for i, g in enumerate(workloads.resnet50_gemms(64, merge=True))}
    idx, g = gemms[name]
    kw = workloads.config_kwargs("resnet50")
    kw["flags"] = (workloads.NI_UPD_NL if "nl" in ni else 0) | workloads.NI_UPD_NOISE
    co, cg = xo.make_config(**kw), xb.make_config(**kw)
    W, X, dY = workloads.layer_tensors_torch(g, seed=idx, device="cuda")
    w_max, xs = 2.0 * float(W.abs().max()), float(X.abs().max())
    bl, dw = 31, 1e-3
    d_range = bl * dw * w_max / (0.01 * xs)
    W0 = W.clone()
    _, pulses = xb.update_pulsed(cg, W, X, dY, w_max, xs, d_range, bl, dw, step=2, want_pulses=True)
    torch.cuda.synchronize()
    rng = np.random.default_rng(idx)
    ks = np.sort(rng.choice(g.K, size=10, replace=False))
    ns = np.sort(rng.choice(g.N, size=10, replace=False))
    ks[0], ks[-1], ns[0], ns[-1] = 0, g.K - 1, 0, g.N - 1
    kt, nt = torch.from_numpy(ks).cuda(), torch.from_numpy(ns).cuda()
    Wo, po = xo.update_pulsed(co, W0[kt][:, nt].cpu().numpy(), X[:, kt].cpu().numpy(), dY[:, nt].cpu().numpy(), w_max, xs, d_range,
                              bl, dw, step=2, want_pulses=True, k_idx=ks, n_idx=ns, K_full=g.K, N_full=g.N)
    assert np.array_equal(pulses[kt][:, nt].cpu().numpy(), po)
    assert np.abs(W[kt][:, nt].cpu().numpy() - Wo).max() <= 2e-7 * w_max
    assert not np.array_equal(Wo, W0[kt][:, nt].cpu().numpy())


def _patch(X, b, oh, ow, k, stride, pad):
    """Patch of output position (b, oh, ow) of the NHWC host array X, index (kh, kw, c), zeros outside."""
    H, W, C = X.shape[1:]
    out = np.zeros((k, k, C), dtype=X.dtype)
    for kh in range(k):
        for kw in range(k):
            ih, iw = oh * stride - pad + kh, ow * stride - pad + kw
            if 0 <= ih < H and 0 <= iw < W:
                out[kh, kw] = X[b, ih, iw]
    return out.reshape(-1)


@pytest.mark.parametrize("name", ["s1b0_3x3", "s2b0_3x3", "conv1_7x7"])
def test_convolution_full_size_sampled(xo, xb, name):
    """ResNet-50 convolutions at batch 64 straight from the NHWC activations (the launch configuration of
    `bench.py --from-images`): sampled output positions, input pixels and weights against the oracle."""
    gemms = {g.name: (i, g) for i, g in enumerate(workloads.resnet50_gemms(64, merge=True))}
    idx, g = gemms[name]
    batch, hw, cin, k, stride, pad = g.conv
    kw = workloads.config_kwargs("resnet50")
    kw["flags"] |= workloads.INPUT_SIGNED if g.signed_input else 0
    co, cg = xo.make_config(**kw), xb.make_config(**kw)
    W, _, dY = workloads.layer_tensors_torch(g, seed=idx, device="cuda")
    X = workloads.image_tensor_torch(g, seed=idx, device="cuda")
    geom = xb.conv_geom(batch, hw, hw, cin, k, k, stride, pad)
    OH, OW = geom.out_h, geom.out_w
    dY4 = dY.view(batch, OH, OW, g.N)
    w_max = 2.0 * float(W.abs().max())
    xs, gs = float(X.abs().max()), float(dY.abs().max())
    planes = xb.tile(cg, W, w_max, 5)
    Y = xb.conv_fwd(cg, planes, X, geom, g.N, w_max, xs)
    dX = xb.conv_bwd(cg, planes, dY4, geom, g.N, w_max, gs)
    W_new = W.clone()
    xb.conv_update(cg, W_new, X, dY4, geom, w_max, 1.0 / w_max, 0.01, 5)
    torch.cuda.synchronize()

    rng = np.random.default_rng(idx)
    Xh, Wh = X.cpu().numpy(), W.cpu().numpy()
    U = xo.planes(co, Wh, w_max, 5)
    # forward: corner positions (padding) and random ones
    pos = [(0, 0, 0), (batch - 1, OH - 1, OW - 1), (1, 0, OW - 1)] + \
          [tuple(int(v) for v in (rng.integers(batch), rng.integers(OH), rng.integers(OW))) for _ in range(5)]
    rows = np.stack([_patch(Xh, b, oh, ow, k, stride, pad) for b, oh, ow in pos])
    Yo = xo.rows_parallel(lambda u, x: xo.fwd_planes(co, u, x, w_max, xs), U, rows, 8)
    Yg = np.stack([Y[b, oh, ow].cpu().numpy() for b, oh, ow in pos])
    assert rel_l2(Yg, Yo) <= 1e-3
    # backward: an input pixel adds the errors of every patch that contains it
    dYh = dY4.cpu().numpy()
    pix = [(0, 0, 0), (batch - 1, hw - 1, hw - 1)] + \
          [tuple(int(v) for v in (rng.integers(batch), rng.integers(hw), rng.integers(hw))) for _ in range(3)]
    for b, ih, iw in pix:
        members = []                                          # (output position, kernel position)
        for kh in range(k):
            for kw_ in range(k):
                oy, ox = ih + pad - kh, iw + pad - kw_
                if oy >= 0 and ox >= 0 and oy % stride == 0 and ox % stride == 0 and oy // stride < OH and ox // stride < OW:
                    members.append((oy // stride, ox // stride, kh, kw_))
        errs = np.stack([dYh[b, oh, ow] for oh, ow, _, _ in members])
        cols = xo.rows_parallel(lambda u, x: xo.bwd_planes(co, u, x, w_max, gs), U, errs, 8)
        want = sum(cols[i].reshape(k, k, cin)[kh, kw_].astype(np.float64) for i, (_, _, kh, kw_) in enumerate(members))
        assert rel_l2(dX[b, ih, iw].cpu().numpy(), want) <= 1e-3
    # update: sampled weights; their patch-matrix columns are single (kh, kw, c) planes of the padded image
    k_idx = np.sort(rng.choice(g.K, size=5, replace=False))
    n_idx = np.sort(rng.choice(g.N, size=4, replace=False))
    Xp = np.pad(Xh, ((0, 0), (pad, pad), (pad, pad), (0, 0)))
    cols = []
    for kk in k_idx:
        c, kw_, kh = kk % cin, (kk // cin) % k, (kk // cin) // k
        cols.append(Xp[:, kh:kh + stride * OH:stride, kw_:kw_ + stride * OW:stride, c].reshape(-1))
    Xsub = np.stack(cols, axis=1)
    Wsub = Wh[np.ix_(k_idx, n_idx)]
    Wo = xo.update(co, Wsub, Xsub, dY[:, torch.from_numpy(n_idx).cuda()].cpu().numpy(), w_max, 1.0 / w_max, 0.01, step=5,
                   k_idx=k_idx, n_idx=n_idx, N_full=g.N)
    Wg = W_new.cpu().numpy()[np.ix_(k_idx, n_idx)]
    assert rel_l2(Wg - Wsub, Wo - Wsub) <= 1e-3
