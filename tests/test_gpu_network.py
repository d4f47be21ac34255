"""A whole training step of a small residual network on the GPU: every kernel call the step makes is
recorded and repeated by the oracle on the same inputs (the GPU run drives the trajectory, so one
flipped ADC code cannot make later comparisons diverge)."""
import ctypes
import math

import numpy as np
import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu


def rel_l2(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def crossbar_outputs_match(got, want, cfg, in_scale, w_max, backward, overlaps=1):
    """Layer outputs against the oracle: an ADC code may differ by one LSB on at most 1e-4 of the
    conversions, and one such flip in the top slice and cycle moves a single output by up to one top-level
    LSB.  So: every element within that step (times the patches a pixel collects), and 1e-3 relative L2
    once the few elements that took a flip are set aside."""
    got, want = np.asarray(got, dtype=np.float64).ravel(), np.asarray(want, dtype=np.float64).ravel()
    q_adc = (1 << (cfg.adc_bits - 1)) - 1
    fs = cfg.adc_fs_bwd if backward else cfg.adc_fs_fwd
    top_shift = cfg.weight_bits - cfg.slice_bits + cfg.input_bits - cfg.stream_bits
    step = fs / q_adc * in_scale * w_max / (((1 << cfg.input_bits) - 1) * ((1 << cfg.weight_bits) - 1)) * 2.0 ** top_shift
    diff = np.abs(got - want)
    assert diff.max() <= 1.01 * step * overlaps
    keep = np.argsort(diff)[:max(1, got.size - 1 - int(1e-3 * got.size))]
    assert np.linalg.norm(diff[keep]) <= 1e-3 * np.linalg.norm(want)
    return True


class Recorder:
    """Stands in for the binding module inside the network driver: forwards every call, keeps copies."""

    def __init__(self, real):
        self.real, self.calls, self.tiled = real, [], {}

    def __getattr__(self, name):
        fn = getattr(self.real, name)
        if not callable(fn) or name in ("make_config", "conv_geom", "planes_bytes", "workspace_bytes",
                                        "conv_workspace_bytes", "lib", "absmax"):
            return fn

        def wrapped(*args, **kw):
            host = lambda v: v.detach().cpu().numpy().copy() if isinstance(v, torch.Tensor) and v.dtype != torch.uint8 else v
            before = [host(a) for a in args]
            if name == "tile":                        # remember which weights / step a plane buffer holds
                self.tiled[kw["planes"].data_ptr()] = (before[1], args[2], args[3])
            out = fn(*args, **kw)
            torch.cuda.synchronize()
            after = [host(o) for o in out] if isinstance(out, tuple) else host(out)
            self.calls.append((name, args, before, after))
            return out
        return wrapped


def oracle_config(xo, cfg):
    skip = ("struct_size", "abi_version", "dac_lut")
    return xo.make_config(**{f: getattr(cfg, f) for f, _ in type(cfg)._fields_ if f not in skip})


@pytest.mark.parametrize("kind", ["basic_blocks", "bottleneck_blocks", "plain_stack"])
def test_residual_network_step_op_by_op(xo, kind):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from oracle import conv, periph
    from paper_2002_11151_amd import resnet_cifar, resnet_imagenet, sequential, xbar as xb
    kw = workloads.config_kwargs("resnet20")
    kw.update(xbar_rows=64, xbar_cols=64, weight_bits=8)
    kw["adc_fs_fwd"] = kw["adc_fs_bwd"] = workloads.adc_full_scale(64, kw["stream_bits"], kw["slice_bits"])
    B = 3
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1)
    if kind == "basic_blocks":
        net = resnet_cifar.ResNetCifar(kw, batch=B, n_blocks=1, image=12, classes=10, widths=(8, 16, 16), seed=3)
        images = torch.randn((B, 12, 12, 3), generator=gen, device="cuda")
        n_conv, n_conv_bwd = 7, 6
    elif kind == "bottleneck_blocks":
        net = resnet_imagenet.ResNetBottleneck(kw, batch=B, image=24, classes=10, blocks=(1, 2), widths=(4, 8), stem=8,
                                               seed=3)
        images = torch.randn((B, 24, 24, 3), generator=gen, device="cuda")
        n_conv, n_conv_bwd = 1 + 3 * 3 + 2, 3 * 3 + 2                    # stem, 3 blocks of 3, 2 projections
    else:
        spec = [("conv", 8, 3, 1, 1), ("relu",), ("maxpool", 2, 2), ("conv", 16, 3, 1, 1), ("relu",), ("conv", 16, 3, 1, 1),
                ("relu",), ("maxpool", 2, 2), ("flatten",), ("fc", 40), ("relu",), ("fc", 10)]
        net = sequential.Sequential(kw, spec, batch=B, in_shape=(12, 12, 3), seed=3)
        images = torch.randn((B, 12, 12, 3), generator=gen, device="cuda")
        n_conv, n_conv_bwd = 3, 2
    labels = torch.tensor([1, 7, 4], dtype=torch.int32, device="cuda")
    net.calibrate(images, labels)
    rec = Recorder(xb)
    net.ops = rec
    loss = net.train_step(images, labels, 0.05)
    assert np.isfinite(loss.cpu().numpy()).all()

    names = [c[0] for c in rec.calls]
    wanted = ["tile", "conv_fwd", "conv_bwd", "conv_update", "fwd", "bwd", "update", "relu_fwd", "relu_bwd", "softmax_xent"]
    if kind != "plain_stack":
        wanted += ["bn_fwd", "bn_bwd", "add", "avgpool_fwd", "avgpool_bwd", "sgd"]
    wanted += ["shortcut_fwd", "shortcut_bwd"] if kind == "basic_blocks" else ["maxpool_fwd", "maxpool_bwd"]
    for want in wanted:
        assert want in names, want
    assert names.count("conv_fwd") == n_conv and names.count("conv_update") == n_conv
    assert names.count("conv_bwd") == n_conv_bwd

    def geom_tuple(g):
        return g.k_h, g.k_w, g.stride, g.pad

    for name, args, a, out in rec.calls:
        if name in ("conv_fwd", "fwd", "conv_bwd", "bwd"):
            cfg, planes = args[0], args[1]
            W, w_max, step = rec.tiled[planes.data_ptr()]
            co = oracle_config(xo, cfg)
        if name == "conv_fwd":
            g = args[3]
            want = xo.fwd(co, W, conv.im2col(a[2], *geom_tuple(g)), w_max, args[6], step=step)
            assert crossbar_outputs_match(out, want, cfg, args[6], w_max, False), name
        elif name == "fwd":
            assert crossbar_outputs_match(out, xo.fwd(co, W, a[2], w_max, args[5], step=step), cfg, args[5], w_max, False), name
        elif name == "conv_bwd":
            g = args[3]
            cols = xo.bwd(co, W, a[2].reshape(-1, args[4]), w_max, args[6], step=step)
            want = conv.col2im(cols, out.shape, *geom_tuple(g))
            assert crossbar_outputs_match(out, want, cfg, args[6], w_max, True, overlaps=g.k_h * g.k_w), name
        elif name == "bwd":
            assert crossbar_outputs_match(out, xo.bwd(co, W, a[2], w_max, args[5], step=step), cfg, args[5], w_max, True), name
        elif name in ("conv_update", "update"):
            co = oracle_config(xo, args[0])
            W0 = a[1]
            if name == "conv_update":
                X, dY = conv.im2col(a[2], *geom_tuple(args[4])), a[3].reshape(-1, W0.shape[1])
                w_max, gs, lr, step = args[5], args[6], args[7], args[8]
            else:
                X, dY = a[2], a[3]
                w_max, gs, lr, step = args[4], args[5], args[6], args[7]
            want = xo.update(co, W0, X, dY, w_max, gs, lr, step=step)
            got = args[1].detach().cpu().numpy()              # W after the step (each layer is written once)
            assert rel_l2(got - W0, want - W0) <= 1e-3, name
        elif name == "bn_fwd":
            y, mean, invstd = periph.bn_fwd(a[0], a[1], a[2], args[3])
            assert rel_l2(out[0], y) <= 1e-5 and rel_l2(out[1], mean) <= 1e-5 and rel_l2(out[2], invstd) <= 1e-5
        elif name == "bn_bwd":
            dx, dgamma, dbeta = periph.bn_bwd(a[0], a[1], a[2], a[3].astype(np.float64), a[4].astype(np.float64))
            assert rel_l2(out[0], dx) <= 1e-4 and rel_l2(out[1], dgamma) <= 1e-4 and rel_l2(out[2], dbeta) <= 1e-4
        elif name == "relu_fwd":
            assert np.array_equal(out, periph.relu_fwd(a[0]).astype(np.float32))
        elif name == "relu_bwd":
            assert np.array_equal(out, periph.relu_bwd(a[0], a[1]).astype(np.float32))
        elif name == "add":
            assert np.array_equal(out, a[0] + a[1])
        elif name == "avgpool_fwd":
            assert rel_l2(out, periph.avgpool_fwd(a[0])) <= 1e-6
        elif name == "avgpool_bwd":
            assert rel_l2(out, periph.avgpool_bwd(a[0], args[1])) <= 1e-6
        elif name == "shortcut_fwd":
            assert np.array_equal(out, periph.shortcut_fwd(a[0], args[1], args[2]).astype(np.float32))
        elif name == "shortcut_bwd":
            assert np.array_equal(out, periph.shortcut_bwd(a[0], args[1], args[2]).astype(np.float32))
        elif name == "maxpool_fwd":
            g = args[1]
            y, arg = periph.maxpool_fwd(a[0], g.k_h, g.stride, g.pad)
            assert np.array_equal(out[0], y.astype(np.float32)) and np.array_equal(out[1], arg)
        elif name == "maxpool_bwd":
            g = args[2]
            assert rel_l2(out, periph.maxpool_bwd(a[0], a[1], (g.batch, g.in_h, g.in_w, g.in_c))) <= 1e-6
        elif name == "softmax_xent":
            lo, dz = periph.softmax_xent(a[0], a[1], np.float64(np.float32(args[2])))
            assert rel_l2(out[0], lo) <= 1e-6 and rel_l2(out[1], dz) <= 1e-6


def test_residual_network_learns_a_fixed_batch():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2002_11151_amd import resnet_cifar
    kw = workloads.config_kwargs("resnet20")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    B = 16
    images = torch.randn((B, 16, 16, 3), generator=gen, device="cuda")
    labels = (torch.arange(B, device="cuda") % 10).to(torch.int32)
    net = resnet_cifar.ResNetCifar(kw, batch=B, n_blocks=1, image=16, classes=10, widths=(16, 32, 64), seed=1)
    net.calibrate(images, labels)
    losses = [float(net.train_step(images, labels, 0.05).mean()) for _ in range(30)]
    assert np.isfinite(losses).all()
    assert np.mean(losses[-5:]) < 0.8 * np.mean(losses[:3]), losses       # 8-bit ADCs, wire drops, write noise: slow but steady


def test_perceptron_learns_with_pulse_level_updates():
    """Second benchmark configuration (784-500-10 perceptron) trained pulse by pulse: stochastic pulse trains on
    non-ideal devices drive the loss of a fixed batch down like the aggregate write does."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2002_11151_amd import sequential
    kw = workloads.config_kwargs("mlp")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(3)
    B = 64
    images = torch.rand((B, 784), generator=gen, device="cuda")
    labels = (torch.arange(B, device="cuda") % 10).to(torch.int32)
    runs = {}
    for kind in ("aggregate", "pulsed"):
        net = sequential.Sequential(kw, sequential.mlp_spec((500,), 10), batch=B, in_shape=(784,), signed_input=False, seed=2)
        if kind == "pulsed":
            net.pulse = dict(bl=31, dw_min=1e-3)
        net.calibrate(images, labels)
        runs[kind] = [float(net.train_step(images, labels, 0.01).mean()) for _ in range(60)]
        assert np.isfinite(runs[kind]).all()
    for kind, losses in runs.items():
        assert max(losses) < 1.1 * losses[0], (kind, losses)                      # no excursion
        assert np.mean(losses[-5:]) < 0.85 * losses[0], (kind, losses)            # 2.45 -> about 1.7 .. 1.9
    # same mean update and the same noise per written change by construction: the runs stay together
    assert abs(np.mean(runs["pulsed"][-5:]) - np.mean(runs["aggregate"][-5:])) < 0.12 * runs["aggregate"][0]

def test_perceptron_learns_with_coded_pulses():
    """Deterministic time-coded pulses (5 frames x 6 sub-slots): the errors use their calibrated range, the pulse
    size follows from the learning rate; values below half a level write nothing, so the loss falls more slowly than
    with stochastic trains (2.45 -> about 2.0 after 60 steps against 1.9)."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2002_11151_amd import sequential, xbar as xb
    kw = workloads.config_kwargs("mlp")
    kw["flags"] |= xb.PULSE_CODED
    gen = torch.Generator(device="cuda")
    gen.manual_seed(3)
    B = 64
    images = torch.rand((B, 784), generator=gen, device="cuda")
    labels = (torch.arange(B, device="cuda") % 10).to(torch.int32)
    net = sequential.Sequential(kw, sequential.mlp_spec((500,), 10), batch=B, in_shape=(784,), signed_input=False, seed=2)
    net.pulse = dict(bl=31)
    net.calibrate(images, labels)
    losses = [float(net.train_step(images, labels, 0.01).mean()) for _ in range(60)]
    assert np.isfinite(losses).all() and max(losses) < 1.1 * losses[0], losses
    assert np.mean(losses[-5:]) < 0.9 * losses[0], losses


def test_perceptron_learns_with_magnitude_coded_pulses_and_with_device_pairs():
    """The two update variants that complete Sec. IV-C's list on the same fixed batch: magnitude-coded pulses (one
    pulse per sample and line with 8 height levels; errors on their calibrated range, quantum from the learning
    rate) and the aggregate write with the two devices of every weight as states of their own."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2002_11151_amd import sequential, xbar as xb
    gen = torch.Generator(device="cuda")
    gen.manual_seed(3)
    B = 64
    images = torch.rand((B, 784), generator=gen, device="cuda")
    labels = (torch.arange(B, device="cuda") % 10).to(torch.int32)
    runs = {}
    for kind in ("aggregate", "pairs", "magnitude"):
        kw = workloads.config_kwargs("mlp")
        if kind == "magnitude":
            kw["flags"] |= xb.PULSE_MAGNITUDE
        net = sequential.Sequential(kw, sequential.mlp_spec((500,), 10), batch=B, in_shape=(784,), signed_input=False, seed=2)
        if kind == "magnitude":
            net.pulse = dict(bl=8)
        net.pair_devices = kind == "pairs"
        net.calibrate(images, labels)
        runs[kind] = [float(net.train_step(images, labels, 0.01).mean()) for _ in range(60)]
        assert np.isfinite(runs[kind]).all() and max(runs[kind]) < 1.1 * runs[kind][0], (kind, runs[kind])
        if kind == "pairs":       # the weights the generator sees are the pairs' differences
            for layer in net.layers:
                gp, gn = layer.pair
                assert torch.equal(layer.W, (layer.w_max * (gp.double() - gn.double())).float())
                assert float(gp.min()) >= 0.0 and float(gp.max()) <= 1.0 and float(gn.min()) >= 0.0 and float(gn.max()) <= 1.0
    assert np.mean(runs["aggregate"][-5:]) < 0.85 * runs["aggregate"][0]
    # same mean change, and per weight the same noise variance as the effective device: the runs stay together
    assert abs(np.mean(runs["pairs"][-5:]) - np.mean(runs["aggregate"][-5:])) < 0.12 * runs["aggregate"][0], runs["pairs"]
    # 8 levels per line: values below half a level write nothing, so slower than the aggregate write
    assert np.mean(runs["magnitude"][-5:]) < 0.95 * runs["magnitude"][0], runs["magnitude"]


def test_residual_network_learns_with_pulse_level_updates():
    """Convolution layers written pulse by pulse (every output position one sample of the pulse scheme): with
    the write non-linearity and no write noise the loss of a fixed batch falls as under the aggregate write."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2002_11151_amd import resnet_cifar
    kw = workloads.config_kwargs("resnet20")
    kw["upd_noise_gamma"] = 0.0
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    B = 16
    images = torch.randn((B, 16, 16, 3), generator=gen, device="cuda")
    labels = (torch.arange(B, device="cuda") % 10).to(torch.int32)
    runs = {}
    for kind in ("aggregate", "pulsed"):
        net = resnet_cifar.ResNetCifar(kw, batch=B, n_blocks=1, image=16, classes=10, widths=(16, 32, 64), seed=1)
        if kind == "pulsed":
            net.pulse = dict(bl=31, dw_min=1e-3)
        net.calibrate(images, labels)
        runs[kind] = [float(net.train_step(images, labels, 0.05).mean()) for _ in range(30)]
        assert np.isfinite(runs[kind]).all()
        assert np.mean(runs[kind][-5:]) < 0.6 * runs[kind][0], (kind, runs[kind])        # 2.74 -> about 1.1
    assert abs(np.mean(runs["pulsed"][-5:]) - np.mean(runs["aggregate"][-5:])) < 0.3


@pytest.mark.parametrize("variant", ["offset", "per_array", "all_paths"])
def test_perceptron_learns_under_variants(variant):
    """The same perceptron with the errors offset-coded (one phase), with one converter per array (range twice as
    wide: an array alone carries its off-state current) and with the all-paths wire model: each learns the fixed
    batch like the default configuration does (2.45 -> about 1.7 .. 1.8 in 60 steps)."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2002_11151_amd import sequential
    kw = workloads.config_kwargs("mlp")
    if variant == "offset":
        kw["flags"] |= workloads.INPUT_OFFSET
    elif variant == "per_array":
        kw["flags"] |= workloads.ADC_PER_ARRAY
        kw["adc_fs_fwd"] *= 2.0
        kw["adc_fs_bwd"] *= 2.0
    else:
        kw["flags"] = (kw["flags"] & ~workloads.NI_WIRE_AAM) | workloads.NI_WIRE_AAM2
    gen = torch.Generator(device="cuda")
    gen.manual_seed(3)
    B = 64
    images = torch.rand((B, 784), generator=gen, device="cuda")
    labels = (torch.arange(B, device="cuda") % 10).to(torch.int32)
    net = sequential.Sequential(kw, sequential.mlp_spec((500,), 10), batch=B, in_shape=(784,), signed_input=False, seed=2)
    net.calibrate(images, labels)
    losses = [float(net.train_step(images, labels, 0.01).mean()) for _ in range(60)]
    assert np.isfinite(losses).all()
    assert max(losses) < 1.1 * losses[0] and np.mean(losses[-5:]) < 0.85 * losses[0], losses

def test_sigmoid_perceptron_step():
    """A perceptron with sigmoid hidden units (Sec. IV-B names sigmoid among the digital peripherals): one training
    step runs and lowers the loss of a fixed batch over a few steps."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2002_11151_amd import sequential
    kw = workloads.config_kwargs("mlp")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(4)
    B = 64
    images = torch.rand((B, 784), generator=gen, device="cuda")
    labels = (torch.arange(B, device="cuda") % 10).to(torch.int32)
    net = sequential.Sequential(kw, sequential.mlp_spec((500,), 10, activation="sigmoid"), batch=B, in_shape=(784,),
                                signed_input=False, seed=2)
    net.calibrate(images, labels)
    losses = [float(net.train_step(images, labels, 0.02).mean()) for _ in range(60)]
    assert np.isfinite(losses).all() and np.mean(losses[-5:]) < 0.95 * losses[0], losses

def test_converter_ranges_from_current_statistics():
    """Sec. IV-B: the maximum current through the ADCs is data dependent and comes from output statistics.
    `calibrate(..., adc_quantile=q)` measures the column currents of every layer (statistics pass on the device)
    and sets the ranges; the ranges come out tighter than the worst-case rule and training gets better."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2002_11151_amd import resnet_cifar
    kw = workloads.config_kwargs("resnet20")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    B = 16
    images = torch.randn((B, 16, 16, 3), generator=gen, device="cuda")
    labels = (torch.arange(B, device="cuda") % 10).to(torch.int32)
    final = {}
    for q in (None, 0.999):
        net = resnet_cifar.ResNetCifar(kw, batch=B, n_blocks=1, image=16, classes=10, widths=(16, 32, 64), seed=1)
        net.calibrate(images, labels, adc_quantile=q)
        if q is not None:
            for layer in net.layers:
                for fs in (layer.cfg.adc_fs_fwd, layer.cfg.adc_fs_bwd):
                    assert 0 < fs <= kw["adc_fs_fwd"] and math.log2(fs) == int(math.log2(fs))       # a power of two, not wider
            assert any(layer.cfg.adc_fs_bwd < kw["adc_fs_bwd"] for layer in net.layers)
            assert all(layer.x_scale > 0 and layer.g_scale > 0 for layer in net.layers)
        losses = [float(net.train_step(images, labels, 0.05).mean()) for _ in range(30)]
        assert np.isfinite(losses).all()
        final[q] = float(np.mean(losses[-5:]))
    assert final[0.999] < final[None] + 0.1, final          # measured here: 1.33 against 1.87

def test_interpolated_circuit_model_in_training():
    """Sec. IV-D: the circuit-level crossbar model is run every L iterations and its stored distortion profile is
    reused in between.  The driver does that when the layers use the stored-profile wire model; the profile is
    computed once per L steps and the network learns the fixed batch."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2002_11151_amd import sequential, xbar as xb

    class Counting:
        def __init__(self):
            self.solves = 0

        def __getattr__(self, name):
            if name == "fcm_profile":
                self.solves += 1
            return getattr(xb, name)

    kw = workloads.config_kwargs("mlp")
    kw["flags"] = (kw["flags"] & ~workloads.NI_WIRE_AAM) | workloads.NI_WIRE_PROFILE
    gen = torch.Generator(device="cuda")
    gen.manual_seed(3)
    B = 64
    images = torch.rand((B, 784), generator=gen, device="cuda")
    labels = (torch.arange(B, device="cuda") % 10).to(torch.int32)
    net = sequential.Sequential(kw, sequential.mlp_spec((500,), 10), batch=B, in_shape=(784,), signed_input=False, seed=2)
    net.fcm_every = 10
    net.calibrate(images, labels)
    net.ops = Counting()
    losses = [float(net.train_step(images, labels, 0.01).mean()) for _ in range(40)]
    assert net.ops.solves == 2 * 4                              # two layers, steps 0, 10, 20, 30
    assert all(0.0 <= float(layer.profile.min()) and float(layer.profile.max()) < 0.5 for layer in net.layers)
    assert np.isfinite(losses).all() and np.mean(losses[-5:]) < 0.9 * losses[0], losses

@pytest.mark.parametrize("kind", ["perceptron", "residual", "residual_pulsed"])
def test_training_steps_from_a_hip_graph(kind):
    """A captured training step replays as the following steps: the device-side step counter gives every replay
    its own device variation and write noise, and weights and losses equal those of eagerly run steps bit for bit."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2002_11151_amd import resnet_cifar, sequential
    gen = torch.Generator(device="cuda")
    gen.manual_seed(11)
    if kind == "perceptron":
        kw = workloads.config_kwargs("mlp")
        kw["flags"] |= workloads.NI_VARIATION
        kw["var_sigma"] = 0.05
        B = 32
        batches = [torch.rand((B, 784), generator=gen, device="cuda") for _ in range(4)]
        make = lambda: sequential.Sequential(kw, sequential.mlp_spec((500,), 10), batch=B, in_shape=(784,), signed_input=False, seed=2)
    else:
        kw = workloads.config_kwargs("resnet20")
        B = 8
        batches = [torch.randn((B, 16, 16, 3), generator=gen, device="cuda") for _ in range(4)]
        make = lambda: resnet_cifar.ResNetCifar(kw, batch=B, n_blocks=1, image=16, classes=10, widths=(16, 32, 64), seed=1)
    labels = [((torch.arange(B, device="cuda") + i) % 10).to(torch.int32) for i in range(4)]
    eager, graphed = make(), make()
    if kind == "residual_pulsed":        # pulse trains and per-pulse noise are keyed by the step as well
        eager.pulse = graphed.pulse = dict(bl=31, dw_min=1e-3)
    eager.calibrate(batches[0], labels[0])
    graphed.calibrate(batches[0], labels[0])
    want = [eager.train_step(x, l, 0.02).clone() for x, l in zip(batches, labels)]
    got = [graphed.capture(batches[0], labels[0], 0.02).clone()]
    for x, l in zip(batches[1:], labels[1:]):
        torch.cuda.synchronize()                                  # eager work and synchronisation between the replays
        got.append(graphed.replay(x, l).clone())
    torch.cuda.synchronize()
    for a, b in zip(got, want):
        assert torch.equal(a, b)
    for la, lb in zip(graphed.layers, eager.layers):
        assert torch.equal(la.W, lb.W)
    assert graphed.step_no == eager.step_no == 4
    assert not torch.equal(want[0], want[1])


def test_layers_of_equal_shape_draw_their_own_random_numbers():
    """Device variation, write noise and pulse trains are keyed by (seed, stream, step, element): two layers of
    one network with the same shape must not see the same draws at the same step, so every layer has a seed of
    its own."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2002_11151_amd import sequential, xbar as xb
    kw = workloads.config_kwargs("mlp")
    kw.update(flags=kw["flags"] | workloads.NI_VARIATION, var_sigma=0.1, stream_bits=1)
    kw["adc_fs_fwd"] = kw["adc_fs_bwd"] = workloads.adc_full_scale(128, 1, 2)
    net = sequential.Sequential(kw, [("fc", 48), ("fc", 48), ("fc", 48)], batch=8, in_shape=(48,), seed=5)
    first, second = net.layers[1], net.layers[2]                       # both 48 x 48, both with signed inputs
    assert (first.K, first.N) == (second.K, second.N) and first.cfg.flags == second.cfg.flags
    assert first.cfg.seed != second.cfg.seed
    gen = torch.Generator(device="cuda")
    gen.manual_seed(2)
    X = torch.randn((8, 48), generator=gen, device="cuda")
    dY = torch.randn((8, 48), generator=gen, device="cuda") * 0.01
    W = first.W.clone()
    w_max = 2.0 * float(W.abs().max())

    def passes(cfg):
        planes = xb.tile(cfg, W, w_max, 7)
        Y = xb.fwd(cfg, planes, X, 48, w_max, 4.0)                      # device variation of step 7
        Wn = xb.update(cfg, W.clone(), X, dY, w_max, 1.0 / w_max, 0.01, 7)      # write noise of step 7
        return Y, Wn

    Y1, W1 = passes(first.cfg)
    Y1b, W1b = passes(first.cfg)
    Y2, W2 = passes(second.cfg)
    torch.cuda.synchronize()
    assert torch.equal(Y1, Y1b) and torch.equal(W1, W1b)                # same key, same draws
    assert not torch.equal(Y1, Y2) and not torch.equal(W1, W2)          # another layer, other draws
    # the noise fields are unrelated, not shifted copies: their correlation is that of independent draws
    n1, n2 = (W1 - W).flatten().double(), (W2 - W).flatten().double()
    corr = float(torch.dot(n1 - n1.mean(), n2 - n2.mean()) / (n1.std() * n2.std() * (n1.numel() - 1)))
    assert abs(corr) < 0.1
