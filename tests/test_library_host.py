"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the header
declares, validates parameter structs and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def xb():
    from paper_2002_11151_amd import xbar
    if not os.path.exists(xbar.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    xbar.lib()
    return xbar


def test_exports_every_declared_symbol(xb):
    header = open(os.path.join(ROOT, "include", "xbar.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(xbar_[a-z_]+)\s*\(", header))
    assert {"xbar_fwd", "xbar_bwd", "xbar_update", "xbar_tile", "xbar_config_validate", "xbar_planes_bytes",
            "xbar_workspace_bytes", "xbar_strerror", "xbar_abi_version", "xbar_trace_next_vmm", "xbar_probe_mfma_rate"} <= names
    lib = C.CDLL(xb.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n


def test_struct_layout_matches(xb):
    # the library checks struct_size itself: a good struct validates, a truncated one does not
    c = xb.make_config()
    assert xb.validate(c) == 0
    c.struct_size -= 4
    assert xb.validate(c) == -1
    c = xb.make_config()
    c.abi_version = 99
    assert xb.validate(c) == -1


@pytest.mark.parametrize("kw", [
    dict(xbar_rows=60), dict(xbar_rows=8), dict(xbar_cols=512), dict(weight_bits=7, slice_bits=2),
    dict(weight_bits=32, slice_bits=2), dict(slice_bits=5, weight_bits=10), dict(input_bits=9),
    dict(input_bits=8, stream_bits=3), dict(stream_bits=0), dict(adc_bits=1), dict(adc_bits=17),
    dict(flags=1 << 13), dict(flags=2048 | 4096), dict(flags=512 | 256), dict(flags=512, adc_bits=16), dict(flags=256, adc_curve=[0.0] * 8 + [1.0, 0.5] + [1.0] * 7),
    dict(flags=256, adc_curve=[-1.5] + [0.0] * 16), dict(flags=2 | 4), dict(flags=2 | 128), dict(flags=4 | 128), dict(r_min=0.0), dict(r_min=2e6), dict(r_max=float("nan")),
    dict(r_row=-1.0), dict(var_sigma=float("inf")), dict(adc_fs_fwd=0.0), dict(adc_fs_bwd=-3.0),
    dict(upd_noise_gamma=-1.0),
])
def test_validate_rejects(xb, kw):
    assert xb.validate(xb.make_config(**kw)) == -1


@pytest.mark.parametrize("kw", [
    dict(), dict(xbar_rows=128, xbar_cols=256, weight_bits=16), dict(slice_bits=1, weight_bits=16),
    dict(stream_bits=8), dict(slice_bits=4, weight_bits=16, adc_bits=16), dict(flags=127 & ~4),
    dict(xbar_rows=16, xbar_cols=48), dict(flags=128 | 1 | 8 | 16 | 64), dict(flags=256),
    dict(flags=256, adc_curve=[-1.0] * 9 + [1.0] * 8), dict(flags=512), dict(flags=512 | 128 | 1 | 32, adc_bits=15), dict(flags=1024), dict(flags=1024 | 64 | 512 | 2), dict(flags=4096 | 8 | 16),
])
def test_validate_accepts(xb, kw):
    assert xb.validate(xb.make_config(**kw)) == 0


def test_plane_terms_follow_the_converter(xb):
    """Terms of the 6-bit planes: 4 or 5, enough that what they leave of a plane value moves few enough
    conversions across a rounding boundary (estimate: converter gain x largest digit x 0.46 x sqrt(rows / 2)
    x what is left): at most 5e-5 of them, and at most the share that keeps layer outputs within 1e-3
    (5.6e-8 gain^2 rows: a coarse converter's codes weigh more).  Ideal arrays need 1; 5 with a converter per array."""
    import workloads
    base = dict(xbar_rows=128, xbar_cols=128, weight_bits=16, slice_bits=2, input_bits=8, stream_bits=1,
                adc_fs_fwd=64.0, adc_fs_bwd=64.0)
    for bits, flags, want in ((4, xb.NI_WIRE_AAM, 5), (6, xb.NI_WIRE_AAM, 5), (8, xb.NI_WIRE_AAM, 4), (10, xb.NI_WIRE_AAM, 4), (12, xb.NI_WIRE_AAM, 5),
                              (8, xb.NI_WIRE_AAM | xb.NI_VARIATION, 5), (8, 0, 1), (16, 0, 1),
                              (8, xb.ADC_PER_ARRAY, 5), (4, xb.ADC_PER_ARRAY | xb.NI_WIRE_AAM, 5)):
        assert xb.plane_format(xb.make_config(adc_bits=bits, flags=flags, var_sigma=0.1, **base)) == (1, want), (bits, flags)
    # the benchmark configurations
    assert xb.plane_format(xb.make_config(**workloads.config_kwargs("resnet50"))) == (1, 4)
    assert xb.plane_format(xb.make_config(**workloads.config_kwargs("vgg16"))) == (1, 5)
    assert xb.plane_format(xb.make_config(**workloads.config_kwargs("resnet20")))[0] == 0     # cycles of 4 bits: fp16 planes


def test_size_queries(xb):
    pad256 = lambda b: -(-b // 256) * 256
    K, N = 147, 64
    # cycles of 4 bits: fp16 planes.  Forward copy: ceil(K/128) tiles x ceil(N/32) patches x 8 slices x 2 terms
    # x 8 KiB, same for backward
    base = dict(xbar_rows=128, xbar_cols=128, weight_bits=16, slice_bits=2, stream_bits=4)
    c16 = xb.make_config(flags=xb.NI_WIRE_AAM, **base)
    fwd = 2 * 2 * 8 * 2 * 8 * 1024
    bwd = 1 * 5 * 8 * 2 * 8 * 1024
    assert xb.planes_bytes(c16, K, N) == fwd + bwd
    assert xb.planes_bytes(xb.make_config(**base), K, N) == (fwd + bwd) // 2
    for flags in (xb.ADC_PER_ARRAY, xb.ADC_PER_ARRAY | xb.NI_WIRE_AAM):      # arrays apart: two terms even when ideal
        assert xb.planes_bytes(xb.make_config(flags=flags, **base), K, N) == 2 * (fwd + bwd)
    # cycles of 1 or 2 bits: 6-bit planes, 1.5 KiB per 64 rows x 32 columns and term, + 1 KiB behind each copy.
    # Single-path wire model alone: 4 terms; with variation (or arrays apart): 5; ideal arrays: 1
    base = dict(xbar_rows=128, xbar_cols=128, weight_bits=16, slice_bits=2)
    c = xb.make_config(flags=xb.NI_WIRE_AAM, **base)
    frag = lambda terms, arrays=1: ((2 * 2 + 1 * 5) * 8 * terms * 2 * 1536) * arrays + pad256(1024) * 2
    # single-path wire model alone: the table of term codes (2 orientations x 2 signs x 3 digits x 128 x 128
    # words) rides behind the planes
    table = 2 * 2 * 3 * 128 * 128 * 4
    assert xb.planes_bytes(c, K, N) == frag(4) + table
    # any other array non-ideality: every device is computed once into a word of term codes per array, slice and
    # weight, kept behind the planes, from which both copies are packed
    words = lambda arrays=1: pad256(4 * arrays * 8 * K * N)
    assert xb.planes_bytes(xb.make_config(flags=xb.NI_WIRE_AAM | xb.NI_VARIATION, **base), K, N) == frag(5) + words()
    assert xb.planes_bytes(xb.make_config(**base), K, N) == frag(1)
    assert xb.planes_bytes(xb.make_config(flags=xb.ADC_PER_ARRAY, **base), K, N) == frag(5, 2) + words(2)
    # a general DAC level table runs on the fp16 path
    lut = xb.make_config(flags=xb.NI_WIRE_AAM | xb.DAC_LUT, stream_bits=2, dac_lut=[0.0, 0.3, 0.7, 1.0], **base)
    assert xb.planes_bytes(lut, K, N) == fwd + bwd
    all_paths = xb.make_config(flags=xb.NI_WIRE_AAM2, **base)
    assert xb.planes_bytes(all_paths, K, N) == frag(5) + 16 * 8 * K * N + 4 * K * N + words()   # scratch behind the planes
    fwd, bwd = frag(4) // 2, frag(4) // 2
    # offset-binary inputs: the 64-bit sums of the programmed weights per column and per row ride along
    coded = xb.make_config(xbar_rows=128, xbar_cols=128, weight_bits=16, slice_bits=2, flags=xb.NI_WIRE_AAM | xb.INPUT_OFFSET)
    assert xb.planes_bytes(coded, K, N) == fwd + bwd + -(-8 * (K + N) // 256) * 256 + table
    # ... and one phase instead of two: half the staged input of a signed pass
    assert xb.workspace_bytes(coded, xb.OP_BWD, 64, K, N) < xb.workspace_bytes(c, xb.OP_BWD, 64, K, N)
    assert xb.planes_bytes(c, 0, N) == 0 and xb.planes_bytes(c, K, -1) == 0
    for op in (xb.OP_FWD, xb.OP_BWD, xb.OP_UPDATE):
        small, big = xb.workspace_bytes(c, op, 64, K, N), xb.workspace_bytes(c, op, 6400, K, N)
        assert 0 < small <= big
        assert xb.workspace_bytes(c, op, 0, K, N) == 0
    assert xb.workspace_bytes(c, 7, 64, K, N) == 0
    # pulse-level update: trains of a chunk of samples (4 bytes per input and error, at most 64 MiB or 64
    # samples) and the double-precision states between chunks
    pad = lambda b: -(-b // 256) * 256
    assert xb.workspace_bytes(c, xb.OP_UPDATE_PULSED, 100, K, N) == pad(400 * K) + pad(400 * N) + pad(8 * K * N)
    big = xb.workspace_bytes(c, xb.OP_UPDATE_PULSED, 1 << 22, K, N)
    mc_big = ((64 << 20) // (4 * (K + N))) // 64 * 64
    marks = pad(mc_big // 64 * 8 * K * N) + pad(-(-mc_big // 4096) * 8 * K * N)                       # 40 blocks of devices: the marking pass is used
    assert big - pad(8 * K * N) - marks <= (64 << 20) + 512 and big > xb.workspace_bytes(c, xb.OP_UPDATE_PULSED, 100, K, N)
    assert xb.workspace_bytes(c, xb.OP_UPDATE_PULSED, 1 << 22, 2048, 1030) - pad(8 * 2048 * 1030) <= (64 << 20) + 512
    # few devices, many samples (a convolution layer): one mark bit per sample and device on top
    mc = ((64 << 20) // (4 * (144 + 16))) // 64 * 64
    assert xb.workspace_bytes(c, xb.OP_UPDATE_PULSED, 131072, 144, 16) == (
        pad(4 * mc * 144) + pad(4 * mc * 16) + pad(8 * 144 * 16) + pad(-(-mc // 64) * 8 * 144 * 16) + pad(-(-mc // 4096) * 8 * 144 * 16))
    # the marks stay within 256 MiB: 512 x 256 devices take 16384 samples at a time
    assert xb.workspace_bytes(c, xb.OP_UPDATE_PULSED, 20000, 512, 256) == (
        pad(4 * 16384 * 512) + pad(4 * 16384 * 256) + pad(8 * 512 * 256) + pad(256 * 8 * 512 * 256) + pad(4 * 8 * 512 * 256))
    assert xb.workspace_bytes(c, xb.OP_UPDATE_PULSED, 2047, 144, 16) == pad(4 * 2047 * 144) + pad(4 * 2047 * 16) + pad(8 * 144 * 16)
    # circuit-level model: 5 crossbar-sized fp64 vectors per resident block, at most 2048 blocks
    items = 2 * 1 * 8 * 2                                   # (row tiles x column tiles) x slices x arrays
    assert xb.workspace_bytes(c, xb.OP_FCM, 1, K, N) % (5 * 128 * 128 * 8) == 0
    assert items * 5 * 128 * 128 * 8 <= xb.workspace_bytes(c, xb.OP_FCM, 1, K, N) <= 2048 * 5 * 128 * 128 * 8
    assert xb.workspace_bytes(c, xb.OP_FWD, 1 << 20, 1 << 12, 8) > 0      # activations may exceed 2^31 elements
    assert xb.workspace_bytes(c, xb.OP_FWD, 8, 1 << 16, 1 << 15) == 0     # K*N reaches 2^31
    assert xb.workspace_bytes(c, xb.OP_FWD, 1 << 30, 1 << 8, 8) == 0      # M*K reaches 2^38


def test_argument_checks_precede_any_device_work(xb):
    lib = xb.lib()
    c = xb.make_config()
    ok = C.c_void_p(0x1000)          # aligned, never dereferenced: every call below fails validation first
    odd = C.c_void_p(0x1004)
    big = 1 << 40
    assert lib.xbar_tile(C.byref(c), ok, 0, 64, 1.0, 0, None, ok, big, None) == -2
    assert lib.xbar_tile(C.byref(c), odd, 64, 64, 1.0, 0, None, ok, big, None) == -3
    assert lib.xbar_tile(C.byref(c), ok, 64, 64, 1.0, 0, None, None, big, None) == -3
    assert lib.xbar_tile(C.byref(c), ok, 64, 64, 0.0, 0, None, ok, big, None) == -1
    assert lib.xbar_tile(C.byref(c), ok, 64, 64, 1.0, 0, None, ok, 16, None) == -4
    prof = xb.make_config(flags=xb.NI_WIRE_PROFILE)
    assert lib.xbar_tile(C.byref(prof), ok, 64, 64, 1.0, 0, None, ok, big, None) == -3
    for fn in (lib.xbar_fwd, lib.xbar_bwd):
        assert fn(C.byref(c), ok, ok, ok, -1, 64, 64, 1.0, 1.0, ok, big, None, None) == -2
        assert fn(C.byref(c), ok, odd, ok, 4, 64, 64, 1.0, 1.0, ok, big, None, None) == -3
        assert fn(C.byref(c), ok, ok, ok, 4, 64, 64, 1.0, float("nan"), ok, big, None, None) == -1
        assert fn(C.byref(c), ok, ok, ok, 4, 64, 64, 1.0, 1.0, ok, 16, None, None) == -4
        bad = xb.make_config(adc_bits=40)
        assert fn(C.byref(bad), ok, ok, ok, 4, 64, 64, 1.0, 1.0, ok, big, None, None) == -1
    assert lib.xbar_update(C.byref(c), ok, ok, ok, 4, 64, 0, 1.0, 1.0, 0.1, 0, ok, big, None) == -2
    assert lib.xbar_update(C.byref(c), ok, ok, odd, 4, 64, 64, 1.0, 1.0, 0.1, 0, ok, big, None) == -3
    assert lib.xbar_update(C.byref(c), ok, ok, ok, 4, 64, 64, 1.0, 1.0, 0.1, 0, ok, 16, None) == -4
    assert lib.xbar_update(C.byref(c), ok, ok, ok, 4, 64, 64, -1.0, 1.0, 0.1, 0, ok, big, None) == -1
    assert lib.xbar_fcm_profile(C.byref(c), ok, 64, 0, 1.0, 0, ok, ok, big, None) == -2
    assert lib.xbar_fcm_profile(C.byref(c), ok, 64, 64, 1.0, 0, odd, ok, big, None) == -3
    assert lib.xbar_fcm_profile(C.byref(c), ok, 64, 64, float("inf"), 0, ok, ok, big, None) == -1
    assert lib.xbar_fcm_profile(C.byref(c), ok, 64, 64, 1.0, 0, ok, ok, 16, None) == -4
    geom = xb.conv_geom(2, 8, 8, 4, 3, 3, 1, 1)
    assert lib.xbar_conv_fwd(C.byref(c), ok, ok, ok, None, 16, 1.0, 1.0, ok, big, None, None) == -1
    assert lib.xbar_conv_fwd(C.byref(c), ok, odd, ok, C.byref(geom), 16, 1.0, 1.0, ok, big, None, None) == -3
    assert lib.xbar_conv_fwd(C.byref(c), ok, ok, ok, C.byref(geom), 16, 1.0, 1.0, ok, 16, None, None) == -4
    assert lib.xbar_conv_bwd(C.byref(c), ok, ok, ok, C.byref(geom), 16, 1.0, 1.0, ok, 16, None) == -4
    assert lib.xbar_conv_update(C.byref(c), ok, ok, ok, C.byref(geom), 16, 1.0, 1.0, 0.1, 0, ok, 16, None) == -4
    assert xb.conv_workspace_bytes(c, xb.OP_BWD, geom, 16) > xb.conv_workspace_bytes(c, xb.OP_FWD, geom, 16) > 0
    assert lib.xbar_conv_update_pulsed(C.byref(c), ok, ok, ok, C.byref(geom), 16, 1.0, 1.0, 1.0, 31, 1e-3, 0, None, ok, 16, None) == -4
    assert lib.xbar_conv_update_pulsed(C.byref(c), ok, ok, ok, None, 16, 1.0, 1.0, 1.0, 31, 1e-3, 0, None, ok, big, None) == -1
    assert xb.conv_workspace_bytes(c, xb.OP_UPDATE_PULSED, geom, 16) == xb.workspace_bytes(c, xb.OP_UPDATE_PULSED, 2 * 8 * 8, 36, 16)
    geom.out_h = 9                                             # not what stride and padding give
    assert xb.conv_workspace_bytes(c, xb.OP_FWD, geom, 16) == 0
    assert lib.xbar_conv_fwd(C.byref(c), ok, ok, ok, C.byref(geom), 16, 1.0, 1.0, ok, big, None, None) == -2
    geom = xb.conv_geom(2, 8, 8, 4, 3, 3, 1, 1)
    geom.pad = -1
    assert lib.xbar_conv_fwd(C.byref(c), ok, ok, ok, C.byref(geom), 16, 1.0, 1.0, ok, big, None, None) == -2
    geom = xb.conv_geom(2, 2, 2, 4, 5, 5, 1, 0)                # kernel larger than the image
    assert lib.xbar_conv_bwd(C.byref(c), ok, ok, ok, C.byref(geom), 16, 1.0, 1.0, ok, big, None) == -2
    assert lib.xbar_adc_histogram(C.byref(c), ok, ok, 4, 64, 64, 1.0, 2, 0.5, ok, ok, big, None) == -1       # no such pass
    assert lib.xbar_adc_histogram(C.byref(c), ok, ok, 4, 64, 64, 1.0, 0, 0.0, ok, ok, big, None) == -1
    assert lib.xbar_adc_histogram(C.byref(c), ok, ok, 4, 64, 64, 1.0, 0, 0.5, odd, ok, big, None) == -3
    assert lib.xbar_adc_histogram(C.byref(c), ok, ok, 4, 64, 64, 1.0, 1, 0.5, ok, ok, 16, None) == -4
    for code in range(-6, 1):
        assert xb.strerror(code) and "unknown" not in xb.strerror(code)
    assert "unknown" in xb.strerror(-99)


def test_bench_refuses_more_than_one_gpu():
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    run = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert run.returncode != 0 and "one GPU" in run.stderr and run.stdout.strip() == ""


def test_pulse_walk_keeps_its_device_model_at_compile_time():
    """Regression guard.  With the device-model flags tested at run time inside the per-lane pulse walk of the
    4 x 4-devices-per-thread kernel, the compiler (hipcc of ROCm 7.2, -O3) turns the wave-uniform test into a
    lane mask made by a vector compare under the execution mask of the FIRST device's walk and reuses that mask
    register in the walks of the thread's other 15 devices, whose active lanes differ: lanes that had left the first
    walk read as "flag set", so linear devices took the non-linear branch (seen in the generated gfx950 code; wrong
    weights for every device but the first of a thread, pulse counts right).  The walk therefore takes its device model
    as template parameters: no wave-uniform condition is live across the per-lane loops.  The GPU cases
    large_layer_linear / large_layer_noise of test_gpu_parity.py catch the effect; this test keeps the source from
    drifting back."""
    import os
    import re
    src = open(os.path.join(os.path.dirname(__file__), "..", "paper_2002_11151_amd", "csrc", "pulse.hip")).read()
    body = src[src.index("__device__ __forceinline__ double one_pulse("):src.index("// Block = (16 P) x (16 P) devices")]
    assert "if constexpr (NL)" in body and "if constexpr (NOISE)" in body
    assert not re.search(r"a\.flags", body), "one_pulse must not test run-time flags"
    for kernel in ("pulse_apply_kernel", "pulse_walk_kernel"):
        start = src.index("void %s(PulseArgs a)" % kernel)
        end = src.index("\n}\n", start)
        assert not re.search(r"a\.flags", src[start:end]), kernel + " must not test run-time flags in its walk"
