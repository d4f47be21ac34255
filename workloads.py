"""Seeded synthetic workloads: layer-GEMM shape tables and input generators.

Serves the tests, the benchmark and the oracle-side scripts alike and holds none of the method's
arithmetic: only shapes, parameter presets and random tensors.  A layer is a GEMM
Y[M x N] = X[M x K] . W[K x N] with K = fan-in (crossbar rows), N = fan-out (crossbar columns) and
M = batch x output positions after im2col.  The paper's data sets and trained weights are replaced by
random tensors of the same shapes and value distributions.
"""
import math
from collections import namedtuple

import numpy as np

# conv: None for a fully connected layer, else (batch, image size, input channels, kernel, stride, pad)
Gemm = namedtuple("Gemm", "name K N M signed_input count conv", defaults=[None])

# flag bits of the parameter struct (plain numbers, typed here so that this module imports nothing)
NI_VARIATION, NI_WIRE_AAM, NI_WIRE_PROFILE, NI_UPD_NL, NI_UPD_NOISE, DAC_LUT, INPUT_SIGNED, NI_WIRE_AAM2 = (
    1, 2, 4, 8, 16, 32, 64, 128)
ADC_CURVE, ADC_PER_ARRAY, INPUT_OFFSET, PULSE_CODED, PULSE_MAGNITUDE = 256, 512, 1024, 2048, 4096
PAPER_NI = NI_WIRE_AAM | NI_UPD_NL | NI_UPD_NOISE  # wire parasitics + write non-linearity + write noise


def _merge(gemms):
    """Collapses repeated shapes into one entry with a count (keeps first-seen order)."""
    out, pos = [], {}
    for g in gemms:
        key = (g.K, g.N, g.M, g.signed_input, g.conv)
        if key in pos:
            i = pos[key]
            out[i] = out[i]._replace(count=out[i].count + 1)
        else:
            pos[key] = len(out)
            out.append(g)
    return out


def resnet50_gemms(batch=64, merge=False):
    """im2col GEMMs of every convolution of a ResNet-50 (stride on the 3x3 convolution) on
    224x224x3 inputs, plus the 2048->1000 classifier: 54 GEMMs."""
    g = [Gemm("conv1_7x7", 3 * 49, 64, batch * 112 * 112, True, 1, (batch, 224, 3, 7, 2, 3))]
    cin, hw = 64, 56
    for stage, (width, blocks) in enumerate(zip((64, 128, 256, 512), (3, 4, 6, 3))):
        for b in range(blocks):
            stride = 2 if (b == 0 and stage > 0) else 1
            hw_out = hw // stride
            p = "s%db%d" % (stage + 1, b)
            g.append(Gemm(p + "_1x1a", cin, width, batch * hw * hw, False, 1, (batch, hw, cin, 1, 1, 0)))
            g.append(Gemm(p + "_3x3", width * 9, width, batch * hw_out * hw_out, False, 1, (batch, hw, width, 3, stride, 1)))
            g.append(Gemm(p + "_1x1b", width, width * 4, batch * hw_out * hw_out, False, 1, (batch, hw_out, width, 1, 1, 0)))
            if b == 0:
                g.append(Gemm(p + "_down", cin, width * 4, batch * hw_out * hw_out, False, 1, (batch, hw, cin, 1, stride, 0)))
            cin, hw = width * 4, hw_out
    g.append(Gemm("fc", 2048, 1000, batch, False, 1))
    return _merge(g) if merge else g


def resnet20_gemms(batch=128, merge=False):
    """3x3 convolution stack of a CIFAR ResNet-20 (16/32/64 channels) on 32x32x3 inputs + 64->10."""
    g = [Gemm("conv1", 27, 16, batch * 1024, True, 1, (batch, 32, 3, 3, 1, 1))]
    cin, hw = 16, 32
    for stage, width in enumerate((16, 32, 64)):
        for b in range(3):
            stride = 2 if (b == 0 and stage > 0) else 1
            hw_out = hw // stride
            g.append(Gemm("s%db%d_a" % (stage + 1, b), cin * 9, width, batch * hw_out * hw_out, False, 1,
                          (batch, hw, cin, 3, stride, 1)))
            g.append(Gemm("s%db%d_b" % (stage + 1, b), width * 9, width, batch * hw_out * hw_out, False, 1,
                          (batch, hw_out, width, 3, 1, 1)))
            cin, hw = width, hw_out
    g.append(Gemm("fc", 64, 10, batch, False, 1))
    return _merge(g) if merge else g


def vgg16_gemms(batch=128, merge=False):
    """13 3x3 convolutions and 3 fully connected layers of VGG-16 on 224x224x3 inputs."""
    g, cin, hw = [], 3, 224
    for i, (width, reps) in enumerate(((64, 2), (128, 2), (256, 3), (512, 3), (512, 3))):
        for r in range(reps):
            g.append(Gemm("conv%d_%d" % (i + 1, r + 1), cin * 9, width, batch * hw * hw, cin == 3, 1))
            cin = width
        hw //= 2
    g += [Gemm("fc6", 25088, 4096, batch, False, 1), Gemm("fc7", 4096, 4096, batch, False, 1),
          Gemm("fc8", 4096, 1000, batch, False, 1)]
    return _merge(g) if merge else g


def mlp_gemms(batch=128):
    return [Gemm("fc1", 784, 500, batch, False, 1), Gemm("fc2", 500, 10, batch, False, 1)]


def fc256_gemms(batch=64):
    return [Gemm("fc", 256, 256, batch, True, 1)]


def adc_full_scale(rows, stream_bits, slice_bits):
    """Stand-in for the paper's data-dependent ADC range (it collects output statistics over training
    epochs): 3.3 standard deviations of a tile current whose `rows` products pair a uniformly
    distributed input digit with a uniformly distributed, randomly signed device digit, rounded up to
    a power of two.  In units of one input level times one device level."""
    lv, lw = (1 << stream_bits) - 1, (1 << slice_bits) - 1
    ev2 = sum(v * v for v in range(lv + 1)) / (lv + 1.0)
    eu2 = sum(u * u for u in range(lw + 1)) / (lw + 1.0)
    return float(2 ** math.ceil(math.log2(3.3 * math.sqrt(rows * ev2 * eu2))))


def adc_full_scale_from_histogram(hist, bin_width, quantile=0.999):
    """ADC full scale from measured statistics: the smallest power of two that is at least the
    `quantile` of the |column current| distribution (hist[b] = count of rne(|I| / bin_width) == b)."""
    hist = np.asarray(hist, dtype=np.float64)
    cum = np.cumsum(hist)
    b = int(np.searchsorted(cum, quantile * cum[-1]))
    current = max((b + 0.5) * bin_width, bin_width)
    return float(2.0 ** math.ceil(math.log2(current)))


def config_kwargs(name):
    """Parameter presets of the five benchmark configurations (keyword arguments of the config
    constructors of both the library binding and the oracle wrapper)."""
    paper = dict(r_min=1e5, r_max=1e6, v_max=1.0, r_row=1.0, r_col=4.6, r_source=0.0, r_sense=0.0,
                 upd_nl_v=0.01, upd_noise_gamma=5.0, var_sigma=0.0, seed=0)
    presets = {
        "fc256": dict(xbar_rows=64, xbar_cols=64, weight_bits=8, slice_bits=2, input_bits=8, stream_bits=4,
                      adc_bits=8, flags=PAPER_NI),
        "mlp": dict(xbar_rows=128, xbar_cols=128, weight_bits=8, slice_bits=2, input_bits=8, stream_bits=4,
                    adc_bits=8, flags=PAPER_NI),
        "resnet20": dict(xbar_rows=128, xbar_cols=128, weight_bits=16, slice_bits=2, input_bits=8,
                         stream_bits=4, adc_bits=8, flags=PAPER_NI),
        "resnet50": dict(xbar_rows=128, xbar_cols=128, weight_bits=16, slice_bits=2, input_bits=8,
                         stream_bits=1, adc_bits=8, flags=PAPER_NI),
        "vgg16": dict(xbar_rows=256, xbar_cols=256, weight_bits=16, slice_bits=2, input_bits=8,
                      stream_bits=1, adc_bits=6, flags=PAPER_NI | NI_VARIATION, var_sigma=0.1),
    }
    kw = dict(paper)
    kw.update(presets[name])
    kw["adc_fs_fwd"] = adc_full_scale(kw["xbar_rows"], kw["stream_bits"], kw["slice_bits"])
    kw["adc_fs_bwd"] = adc_full_scale(kw["xbar_cols"], kw["stream_bits"], kw["slice_bits"])
    return kw


GEMMS = {"fc256": fc256_gemms, "mlp": mlp_gemms, "resnet20": resnet20_gemms, "resnet50": resnet50_gemms,
         "vgg16": vgg16_gemms}


# ------------------------------------------------------------------------------------------------
# tensors
# ------------------------------------------------------------------------------------------------
def layer_tensors_np(g, seed, w_std=None, grad_std=0.01, m_rows=None):
    """Host tensors of one layer: W ~ N(0, w_std) (He initialisation if w_std is None), X ~ N(0,1)
    (its absolute value when the layer input is unsigned, i.e. after a ReLU), dY ~ N(0, grad_std).
    m_rows limits the number of batch rows generated."""
    rng = np.random.default_rng(seed)
    M = g.M if m_rows is None else min(g.M, m_rows)
    w_std = math.sqrt(2.0 / g.K) if w_std is None else w_std
    W = (rng.standard_normal((g.K, g.N)) * w_std).astype(np.float32)
    X = rng.standard_normal((M, g.K)).astype(np.float32)
    if not g.signed_input:
        X = np.abs(X)
    dY = (rng.standard_normal((M, g.N)) * grad_std).astype(np.float32)
    return W, X, dY


def uniform_inputs_np(M, K, seed, lo, hi):
    rng = np.random.default_rng(seed)
    return rng.uniform(lo, hi, size=(M, K)).astype(np.float32)


def layer_tensors_torch(g, seed, device, w_std=None, grad_std=0.01):
    """Same distributions as layer_tensors_np, generated directly on `device` with torch's seeded
    generator (used at full benchmark sizes, where the rows the oracle checks are copied back)."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    w_std = math.sqrt(2.0 / g.K) if w_std is None else w_std
    W = torch.randn((g.K, g.N), generator=gen, device=device, dtype=torch.float32) * w_std
    X = torch.randn((g.M, g.K), generator=gen, device=device, dtype=torch.float32)
    if not g.signed_input:
        X = X.abs_()
    dY = torch.randn((g.M, g.N), generator=gen, device=device, dtype=torch.float32) * grad_std
    return W, X, dY


def image_tensor_torch(g, seed, device):
    """NHWC input image of a convolution layer, same value distribution as the rows of layer_tensors_torch."""
    import torch
    batch, hw, cin, _, _, _ = g.conv
    gen = torch.Generator(device=device)
    gen.manual_seed(seed + 1000003)
    X = torch.randn((batch, hw, hw, cin), generator=gen, device=device, dtype=torch.float32)
    return X if g.signed_input else X.abs_()


def macs(g, n_slices, n_cycles, signed_phases=2):
    """Emulated crossbar MACs of one layer: every (slice, cycle, phase) pass counts, a differential
    pair counts once; the update counts the plain outer-product MACs.  Signed inputs take two phases,
    or one when they are streamed as offset-binary codes."""
    base = g.M * g.K * g.N
    fwd = base * n_slices * n_cycles * (signed_phases if g.signed_input else 1)
    bwd = base * n_slices * n_cycles * signed_phases
    return dict(fwd=fwd, bwd=bwd, upd=base, logical=3 * base)
