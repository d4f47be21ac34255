"""Thin binding of the C-ABI library (include/xbar.h): argument marshalling only.

Every step of the path runs in the HIP kernels of libxbar.so; torch is used for device memory and
for the current stream.  There is no CPU fallback: if the library is missing, every call raises.
"""
import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libxbar.so")

(NI_VARIATION, NI_WIRE_AAM, NI_WIRE_PROFILE, NI_UPD_NL, NI_UPD_NOISE, DAC_LUT, INPUT_SIGNED, NI_WIRE_AAM2, ADC_CURVE,
 ADC_PER_ARRAY, INPUT_OFFSET, PULSE_CODED) = (1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024, 2048)
PULSE_MAGNITUDE = 4096
OP_FWD, OP_BWD, OP_UPDATE, OP_FCM, OP_UPDATE_PULSED = 0, 1, 2, 3, 4
ABI_VERSION = 2


class XbarError(RuntimeError):
    pass


class Config(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("abi_version", C.c_uint32),
        ("xbar_rows", C.c_int32), ("xbar_cols", C.c_int32),
        ("weight_bits", C.c_int32), ("slice_bits", C.c_int32),
        ("input_bits", C.c_int32), ("stream_bits", C.c_int32),
        ("adc_bits", C.c_int32), ("flags", C.c_uint32),
        ("r_min", C.c_float), ("r_max", C.c_float), ("v_max", C.c_float),
        ("r_row", C.c_float), ("r_col", C.c_float),
        ("r_source", C.c_float), ("r_sense", C.c_float),
        ("var_sigma", C.c_float),
        ("upd_nl_v", C.c_float), ("upd_noise_gamma", C.c_float),
        ("adc_fs_fwd", C.c_float), ("adc_fs_bwd", C.c_float),
        ("dac_lut", C.c_float * 16),
        ("adc_curve", C.c_float * 17),
        ("seed", C.c_uint64),
    ]


class ConvGeom(C.Structure):
    _fields_ = [("batch", C.c_int32), ("in_h", C.c_int32), ("in_w", C.c_int32), ("in_c", C.c_int32),
                ("k_h", C.c_int32), ("k_w", C.c_int32), ("stride", C.c_int32), ("pad", C.c_int32),
                ("out_h", C.c_int32), ("out_w", C.c_int32)]


def conv_geom(batch, in_h, in_w, in_c, k_h, k_w, stride=1, pad=0):
    """xbar_conv_geom with the output size filled in."""
    return ConvGeom(batch, in_h, in_w, in_c, k_h, k_w, stride, pad,
                    (in_h + 2 * pad - k_h) // stride + 1, (in_w + 2 * pad - k_w) // stride + 1)


def make_config(**kw):
    """Parameter struct with the values the paper states (Sec. V, Sec. VI-B) unless overridden."""
    c = Config()
    c.struct_size = C.sizeof(Config)
    c.abi_version = ABI_VERSION
    d = dict(xbar_rows=64, xbar_cols=64, weight_bits=8, slice_bits=2, input_bits=8, stream_bits=1,
             adc_bits=8, flags=0, r_min=1e5, r_max=1e6, v_max=1.0, r_row=1.0, r_col=4.6, r_source=0.0,
             r_sense=0.0, var_sigma=0.0, upd_nl_v=0.01, upd_noise_gamma=5.0, adc_fs_fwd=64.0,
             adc_fs_bwd=64.0, seed=0)
    d.update(kw)
    lut = d.pop("dac_lut", None)
    curve = d.pop("adc_curve", None)
    for k, v in d.items():
        setattr(c, k, v)
    for i in range(17):
        c.adc_curve[i] = curve[i] if curve is not None else -1.0 + i / 8.0
    levels = max(1, (1 << max(0, min(4, c.stream_bits))) - 1)
    for i in range(16):
        c.dac_lut[i] = (lut[i] if lut is not None and i < len(lut) else (i / levels if i <= levels else 0.0))
    return c


_lib = None

_SIGNATURES = {
    "xbar_abi_version": (C.c_uint32, []),
    "xbar_strerror": (C.c_char_p, [C.c_int]),
    "xbar_config_validate": (C.c_int, [C.POINTER(Config)]),
    "xbar_planes_bytes": (C.c_size_t, [C.POINTER(Config), C.c_int, C.c_int]),
    "xbar_workspace_bytes": (C.c_size_t, [C.POINTER(Config), C.c_int, C.c_int, C.c_int, C.c_int]),
    "xbar_tile": (C.c_int, [C.POINTER(Config), C.c_void_p, C.c_int, C.c_int, C.c_float, C.c_uint64, C.c_void_p,
                            C.c_void_p, C.c_size_t, C.c_void_p]),
    "xbar_fwd": (C.c_int, [C.POINTER(Config), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int,
                           C.c_float, C.c_float, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]),
    "xbar_bwd": (C.c_int, [C.POINTER(Config), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int,
                           C.c_float, C.c_float, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]),
    "xbar_fwd_static": (C.c_int, [C.POINTER(Config), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int,
                                  C.c_float, C.c_float, C.c_void_p]),
    "xbar_plane_format": (C.c_int, [C.POINTER(Config), C.POINTER(C.c_int)]),
    "xbar_adc_range_from_histogram": (C.c_float, [C.c_void_p, C.c_int, C.c_float, C.c_double]),
    "xbar_pulse_slots": (C.c_int, [C.POINTER(Config), C.c_int]),
    "xbar_trace_next_vmm": (None, [C.c_void_p, C.c_void_p]),
    "xbar_set_step_source": (None, [C.c_void_p]),
    "xbar_step_advance": (C.c_int, [C.c_void_p, C.c_void_p]),
    "xbar_probe_mfma_rate": (C.c_int, [C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]),
    "xbar_fcm_profile": (C.c_int, [C.POINTER(Config), C.c_void_p, C.c_int, C.c_int, C.c_float, C.c_uint64, C.c_void_p,
                                   C.c_void_p, C.c_size_t, C.c_void_p]),
    "xbar_conv_workspace_bytes": (C.c_size_t, [C.POINTER(Config), C.c_int, C.POINTER(ConvGeom), C.c_int]),
    "xbar_conv_fwd": (C.c_int, [C.POINTER(Config), C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(ConvGeom), C.c_int,
                                C.c_float, C.c_float, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]),
    "xbar_conv_bwd": (C.c_int, [C.POINTER(Config), C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(ConvGeom), C.c_int,
                                C.c_float, C.c_float, C.c_void_p, C.c_size_t, C.c_void_p]),
    "xbar_conv_update": (C.c_int, [C.POINTER(Config), C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(ConvGeom), C.c_int,
                                   C.c_float, C.c_float, C.c_float, C.c_uint64, C.c_void_p, C.c_size_t, C.c_void_p]),
    "xbar_pair_init": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_float, C.c_void_p]),
    "xbar_update_pair": (C.c_int, [C.POINTER(Config), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                   C.c_int, C.c_int, C.c_float, C.c_float, C.c_float, C.c_uint64, C.c_void_p, C.c_size_t,
                                   C.c_void_p]),
    "xbar_conv_update_pair": (C.c_int, [C.POINTER(Config), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.POINTER(ConvGeom), C.c_int, C.c_float, C.c_float, C.c_float, C.c_uint64,
                                        C.c_void_p, C.c_size_t, C.c_void_p]),
    "xbar_relu_fwd": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "xbar_relu_bwd": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "xbar_sigmoid_fwd": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "xbar_sigmoid_bwd": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "xbar_add": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "xbar_sgd": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_float, C.c_void_p]),
    "xbar_bn_workspace_bytes": (C.c_size_t, [C.c_size_t, C.c_int]),
    "xbar_bn_fwd": (C.c_int, [C.c_void_p] * 6 + [C.c_size_t, C.c_int, C.c_float, C.c_void_p, C.c_size_t, C.c_void_p]),
    "xbar_bn_bwd": (C.c_int, [C.c_void_p] * 8 + [C.c_size_t, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]),
    "xbar_avgpool_fwd": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]),
    "xbar_avgpool_bwd": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]),
    "xbar_maxpool_fwd": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(ConvGeom), C.c_void_p]),
    "xbar_maxpool_bwd": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(ConvGeom), C.c_void_p]),
    "xbar_softmax_xent": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_float,
                                    C.c_void_p]),
    "xbar_shortcut_fwd": (C.c_int, [C.c_void_p, C.c_void_p] + [C.c_int] * 6 + [C.c_void_p]),
    "xbar_shortcut_bwd": (C.c_int, [C.c_void_p, C.c_void_p] + [C.c_int] * 6 + [C.c_void_p]),
    "xbar_absmax": (C.c_int, [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "xbar_adc_histogram": (C.c_int, [C.POINTER(Config), C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_float,
                                     C.c_int, C.c_float, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "xbar_conv_adc_histogram": (C.c_int, [C.POINTER(Config), C.c_void_p, C.c_void_p, C.POINTER(ConvGeom), C.c_int,
                                          C.c_float, C.c_int, C.c_float, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "xbar_update": (C.c_int, [C.POINTER(Config), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int,
                              C.c_float, C.c_float, C.c_float, C.c_uint64, C.c_void_p, C.c_size_t, C.c_void_p]),
    "xbar_update_pulsed": (C.c_int, [C.POINTER(Config), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int,
                                     C.c_float, C.c_float, C.c_float, C.c_int, C.c_float, C.c_uint64, C.c_void_p,
                                     C.c_void_p, C.c_size_t, C.c_void_p]),
    "xbar_conv_update_pulsed": (C.c_int, [C.POINTER(Config), C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(ConvGeom),
                                          C.c_int, C.c_float, C.c_float, C.c_float, C.c_int, C.c_float, C.c_uint64,
                                          C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
}


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise XbarError("libxbar.so is not built (run `python -c 'import __graft_entry__ as g; g.build()'`); "
                            "there is no fallback path")
        _lib = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            f = getattr(_lib, name)
            f.restype, f.argtypes = res, args
        if _lib.xbar_abi_version() != ABI_VERSION:
            raise XbarError("libxbar.so has a different ABI version")
    return _lib


def strerror(code):
    return lib().xbar_strerror(code).decode()


def _check(code):
    if code != 0:
        raise XbarError("xbar error %d: %s" % (code, strerror(code)))


def trace_next_vmm(before, after):
    """xbar_trace_next_vmm: hipEvent_t handles (integers) recorded around the next contraction kernel."""
    lib().xbar_trace_next_vmm(C.c_void_p(before), C.c_void_p(after))


def probe_mfma_rate(mode, iters, scratch):
    """xbar_probe_mfma_rate: enqueue the matrix-instruction probe; returns the flops (multiply + add of every
    product of every instruction) that it issues on its 2048 waves."""
    _check(lib().xbar_probe_mfma_rate(mode, iters, C.c_void_p(scratch.data_ptr()), scratch.numel(), _stream()))
    per_instruction = {0: 16384, 1: 16384, 2: 32768, 3: 32768}.get(mode, 65536)      # 32 x 32 x (16 | 32 | 64)
    per_iteration = 32 if mode >= 5 else 16
    return 2.0 * per_iteration * iters * 2048 * per_instruction


def adc_range_from_histogram(hist, bin_width, quantile):
    """xbar_adc_range_from_histogram: converter range from the counters of adc_histogram (copied to the host)."""
    host = hist.detach().to("cpu", torch.int64).contiguous()
    fs = lib().xbar_adc_range_from_histogram(C.c_void_p(host.data_ptr()), host.numel(), bin_width, quantile)
    if fs <= 0.0:
        raise XbarError("xbar_adc_range_from_histogram: invalid arguments")
    return float(fs)


def pulse_slots(cfg, bl):
    """xbar_pulse_slots: slots of a pulse train that carry pulses (all bl of a stochastic train, frames x sub-slots
    of a coded one)."""
    n = lib().xbar_pulse_slots(C.byref(cfg), bl)
    _check(min(n, 0))
    return n


def plane_format(cfg):
    """xbar_plane_format: (0 = fp16 planes | 1 = 6-bit planes with 4-bit digits, operand terms per plane value)."""
    terms = C.c_int(0)
    fmt = lib().xbar_plane_format(C.byref(cfg), C.byref(terms))
    _check(min(fmt, 0))
    return fmt, terms.value


def validate(cfg):
    return lib().xbar_config_validate(C.byref(cfg))


def planes_bytes(cfg, K, N):
    return lib().xbar_planes_bytes(C.byref(cfg), K, N)


def workspace_bytes(cfg, op, M, K, N):
    return lib().xbar_workspace_bytes(C.byref(cfg), op, M, K, N)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype=torch.float32):
    assert t.is_cuda and t.dtype == dtype and t.is_contiguous(), "need a contiguous %s CUDA tensor" % dtype
    return C.c_void_p(t.data_ptr())


def _buffer(nbytes, buf, device):
    if buf is None:
        buf = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=device)
    assert buf.is_cuda and buf.dtype == torch.uint8 and buf.is_contiguous()
    return buf


def tile(cfg, W, w_max, step=0, profile=None, planes=None):
    """xbar_tile: planes of W[K][N] (float32 CUDA tensor).  Returns the opaque plane buffer."""
    K, N = W.shape
    nbytes = planes_bytes(cfg, K, N)
    if nbytes == 0:
        _check(validate(cfg) or -2)
    planes = _buffer(nbytes, planes, W.device)
    prof = None if profile is None else _dev(profile)
    _check(lib().xbar_tile(C.byref(cfg), _dev(W), K, N, w_max, step, prof, C.c_void_p(planes.data_ptr()),
                           planes.numel(), _stream()))
    return planes


def _codes_shape(cfg, P, T, M, out_cols):
    """[phase][cycle][slice][tile][M][out], with an [array] axis before [tile] when every array has its converter."""
    head = (P, cfg.input_bits // cfg.stream_bits, cfg.weight_bits // cfg.slice_bits)
    return head + ((2,) if cfg.flags & ADC_PER_ARRAY else ()) + (T, M, out_cols)


def _vmm(fn, op, cfg, planes, inp, out_cols, K, N, w_max, in_scale, ws, out, want_codes):
    M = inp.shape[0]
    nbytes = workspace_bytes(cfg, op, M, K, N)
    if nbytes == 0:
        _check(validate(cfg) or -2)
    ws = _buffer(nbytes, ws, inp.device)
    if out is None:
        out = torch.empty((M, out_cols), dtype=torch.float32, device=inp.device)
    codes = None
    if want_codes:
        P = 2 if ((op == OP_BWD or cfg.flags & INPUT_SIGNED) and not cfg.flags & INPUT_OFFSET) else 1
        tile_len = cfg.xbar_cols if op == OP_BWD else cfg.xbar_rows
        lin = N if op == OP_BWD else K
        T = (lin + tile_len - 1) // tile_len
        codes = torch.zeros(_codes_shape(cfg, P, T, M, out_cols), dtype=torch.int16, device=inp.device)
    _check(fn(C.byref(cfg), C.c_void_p(planes.data_ptr()), _dev(inp), _dev(out), M, K, N, w_max, in_scale,
              C.c_void_p(ws.data_ptr()), ws.numel(), None if codes is None else C.c_void_p(codes.data_ptr()),
              _stream()))
    return (out, codes) if want_codes else out


def fwd(cfg, planes, X, N, w_max, x_scale, ws=None, out=None, want_codes=False):
    """xbar_fwd: Y[M][N] from X[M][K] through the planes of tile()."""
    return _vmm(lib().xbar_fwd, OP_FWD, cfg, planes, X, N, X.shape[1], N, w_max, x_scale, ws, out, want_codes)


def fwd_static(cfg, planes, X, N, w_max, x_scale, out):
    """xbar_fwd_static: xbar_fwd with the workspace in the library's static per-GPU array (allocates nothing:
    the caller passes the output tensor)."""
    M, K = X.shape
    assert out.shape == (M, N) and out.dtype == torch.float32 and out.is_contiguous()
    _check(lib().xbar_fwd_static(C.byref(cfg), C.c_void_p(planes.data_ptr()), _dev(X), _dev(out), M, K, N, w_max, x_scale,
                                 _stream()))
    return out


def bwd(cfg, planes, dY, K, w_max, g_scale, ws=None, out=None, want_codes=False):
    """xbar_bwd: dX[M][K] from dY[M][N] through the same planes."""
    return _vmm(lib().xbar_bwd, OP_BWD, cfg, planes, dY, K, K, dY.shape[1], w_max, g_scale, ws, out, want_codes)


def update(cfg, W, X, dY, w_max, grad_scale, lr, step=0, ws=None):
    """xbar_update: W[K][N] in place from X[M][K] and dY[M][N]."""
    K, N = W.shape
    M = X.shape[0]
    assert X.shape == (M, K) and dY.shape == (M, N)
    nbytes = workspace_bytes(cfg, OP_UPDATE, M, K, N)
    if nbytes == 0:
        _check(validate(cfg) or -2)
    ws = _buffer(nbytes, ws, W.device)
    _check(lib().xbar_update(C.byref(cfg), _dev(W), _dev(X), _dev(dY), M, K, N, w_max, grad_scale, lr, step,
                             C.c_void_p(ws.data_ptr()), ws.numel(), _stream()))
    return W


def update_pulsed(cfg, W, X, dY, w_max, x_range, d_range, bl, dw_min, step=0, ws=None, want_pulses=False):
    """xbar_update_pulsed: W[K][N] in place, one sample and one pulse at a time (stochastic pulse trains).
    With want_pulses also returns the signed pulse count of every device (int64 [K][N])."""
    K, N = W.shape
    M = X.shape[0]
    assert X.shape == (M, K) and dY.shape == (M, N)
    nbytes = workspace_bytes(cfg, OP_UPDATE_PULSED, M, K, N)
    if nbytes == 0:
        _check(validate(cfg) or -2)
    ws = _buffer(nbytes, ws, W.device)
    pulses = torch.empty((K, N), dtype=torch.int64, device=W.device) if want_pulses else None
    _check(lib().xbar_update_pulsed(C.byref(cfg), _dev(W), _dev(X), _dev(dY), M, K, N, w_max, x_range, d_range, bl,
                                    dw_min, step, None if pulses is None else C.c_void_p(pulses.data_ptr()),
                                    C.c_void_p(ws.data_ptr()), ws.numel(), _stream()))
    return (W, pulses) if want_pulses else W


def set_step_source(counter):
    """xbar_set_step_source: `counter` is a one-element int64 CUDA tensor whose value is added to every `step`
    argument from now on (None switches it off).  Keep the tensor alive while it is in use."""
    lib().xbar_set_step_source(None if counter is None else C.c_void_p(counter.data_ptr()))


def step_advance(counter):
    """xbar_step_advance: counter += 1 on the current stream."""
    _check(lib().xbar_step_advance(C.c_void_p(counter.data_ptr()), _stream()))


def fcm_profile(cfg, W, w_max, step=0, ws=None, profile=None):
    """xbar_fcm_profile: distortion profile [S_w][2][K][N] of the circuit-level model for W[K][N]."""
    K, N = W.shape
    nbytes = workspace_bytes(cfg, OP_FCM, 1, K, N)
    if nbytes == 0:
        _check(validate(cfg) or -2)
    ws = _buffer(nbytes, ws, W.device)
    if profile is None:
        profile = torch.empty((cfg.weight_bits // cfg.slice_bits, 2, K, N), dtype=torch.float32, device=W.device)
    _check(lib().xbar_fcm_profile(C.byref(cfg), _dev(W), K, N, w_max, step, _dev(profile), C.c_void_p(ws.data_ptr()),
                                  ws.numel(), _stream()))
    return profile


def conv_workspace_bytes(cfg, op, geom, N):
    return lib().xbar_conv_workspace_bytes(C.byref(cfg), op, C.byref(geom), N)


def _conv_ws(cfg, op, geom, N, ws, device):
    nbytes = conv_workspace_bytes(cfg, op, geom, N)
    if nbytes == 0:
        _check(validate(cfg) or -2)
    return _buffer(nbytes, ws, device)


def conv_fwd(cfg, planes, X, geom, N, w_max, x_scale, ws=None, out=None, want_codes=False):
    """xbar_conv_fwd: Y[batch][out_h][out_w][N] from the NHWC tensor X."""
    ws = _conv_ws(cfg, OP_FWD, geom, N, ws, X.device)
    if out is None:
        out = torch.empty((geom.batch, geom.out_h, geom.out_w, N), dtype=torch.float32, device=X.device)
    codes = None
    if want_codes:
        P = 2 if (cfg.flags & INPUT_SIGNED and not cfg.flags & INPUT_OFFSET) else 1
        K, M = geom.k_h * geom.k_w * geom.in_c, geom.batch * geom.out_h * geom.out_w
        T = (K + cfg.xbar_rows - 1) // cfg.xbar_rows
        codes = torch.zeros(_codes_shape(cfg, P, T, M, N), dtype=torch.int16, device=X.device)
    _check(lib().xbar_conv_fwd(C.byref(cfg), C.c_void_p(planes.data_ptr()), _dev(X), _dev(out), C.byref(geom), N, w_max,
                               x_scale, C.c_void_p(ws.data_ptr()), ws.numel(),
                               None if codes is None else C.c_void_p(codes.data_ptr()), _stream()))
    return (out, codes) if want_codes else out


def conv_bwd(cfg, planes, dY, geom, N, w_max, g_scale, ws=None, out=None):
    """xbar_conv_bwd: dX (NHWC, shape of the layer input) from dY[batch][out_h][out_w][N]."""
    ws = _conv_ws(cfg, OP_BWD, geom, N, ws, dY.device)
    if out is None:
        out = torch.empty((geom.batch, geom.in_h, geom.in_w, geom.in_c), dtype=torch.float32, device=dY.device)
    _check(lib().xbar_conv_bwd(C.byref(cfg), C.c_void_p(planes.data_ptr()), _dev(dY), _dev(out), C.byref(geom), N, w_max,
                               g_scale, C.c_void_p(ws.data_ptr()), ws.numel(), _stream()))
    return out


def conv_update(cfg, W, X, dY, geom, w_max, grad_scale, lr, step=0, ws=None):
    """xbar_conv_update: W[k_h k_w in_c][N] in place from the NHWC tensors X and dY."""
    N = W.shape[1]
    ws = _conv_ws(cfg, OP_UPDATE, geom, N, ws, W.device)
    _check(lib().xbar_conv_update(C.byref(cfg), _dev(W), _dev(X), _dev(dY), C.byref(geom), N, w_max, grad_scale, lr, step,
                                  C.c_void_p(ws.data_ptr()), ws.numel(), _stream()))
    return W


def pair_init(W, w_max, Gp=None, Gn=None):
    """xbar_pair_init: the two device states of every weight, placed symmetrically about mid-range."""
    K, N = W.shape
    Gp = torch.empty_like(W) if Gp is None else Gp
    Gn = torch.empty_like(W) if Gn is None else Gn
    _check(lib().xbar_pair_init(_dev(W), _dev(Gp), _dev(Gn), K, N, w_max, _stream()))
    return Gp, Gn


def update_pair(cfg, Gp, Gn, W, X, dY, w_max, grad_scale, lr, step=0, ws=None):
    """xbar_update_pair: the device states Gp, Gn[K][N] in place from X[M][K] and dY[M][N]; W = w_max (Gp - Gn)."""
    K, N = W.shape
    M = X.shape[0]
    assert X.shape == (M, K) and dY.shape == (M, N) and Gp.shape == (K, N) and Gn.shape == (K, N)
    nbytes = workspace_bytes(cfg, OP_UPDATE, M, K, N)
    if nbytes == 0:
        _check(validate(cfg) or -2)
    ws = _buffer(nbytes, ws, W.device)
    _check(lib().xbar_update_pair(C.byref(cfg), _dev(Gp), _dev(Gn), _dev(W), _dev(X), _dev(dY), M, K, N, w_max, grad_scale,
                                  lr, step, C.c_void_p(ws.data_ptr()), ws.numel(), _stream()))
    return W


def conv_update_pair(cfg, Gp, Gn, W, X, dY, geom, w_max, grad_scale, lr, step=0, ws=None):
    """xbar_conv_update_pair: as update_pair for a convolution layer (NHWC tensors X and dY)."""
    N = W.shape[1]
    ws = _conv_ws(cfg, OP_UPDATE, geom, N, ws, W.device)
    _check(lib().xbar_conv_update_pair(C.byref(cfg), _dev(Gp), _dev(Gn), _dev(W), _dev(X), _dev(dY), C.byref(geom), N, w_max,
                                       grad_scale, lr, step, C.c_void_p(ws.data_ptr()), ws.numel(), _stream()))
    return W


def conv_update_pulsed(cfg, W, X, dY, geom, w_max, x_range, d_range, bl, dw_min, step=0, ws=None, want_pulses=False):
    """xbar_conv_update_pulsed: W[k_h k_w in_c][N] in place from the NHWC tensors X and dY, one output
    position and one pulse at a time."""
    K, N = W.shape
    ws = _conv_ws(cfg, OP_UPDATE_PULSED, geom, N, ws, W.device)
    pulses = torch.empty((K, N), dtype=torch.int64, device=W.device) if want_pulses else None
    _check(lib().xbar_conv_update_pulsed(C.byref(cfg), _dev(W), _dev(X), _dev(dY), C.byref(geom), N, w_max, x_range,
                                         d_range, bl, dw_min, step,
                                         None if pulses is None else C.c_void_p(pulses.data_ptr()),
                                         C.c_void_p(ws.data_ptr()), ws.numel(), _stream()))
    return (W, pulses) if want_pulses else W


# ---- digital peripherals -------------------------------------------------------------------------
def relu_fwd(x, out=None):
    out = torch.empty_like(x) if out is None else out
    _check(lib().xbar_relu_fwd(_dev(x), _dev(out), x.numel(), _stream()))
    return out


def sigmoid_fwd(x, out=None):
    out = torch.empty_like(x) if out is None else out
    _check(lib().xbar_sigmoid_fwd(_dev(x), _dev(out), x.numel(), _stream()))
    return out


def sigmoid_bwd(y, dy, out=None):
    out = torch.empty_like(y) if out is None else out
    _check(lib().xbar_sigmoid_bwd(_dev(y), _dev(dy), _dev(out), y.numel(), _stream()))
    return out


def relu_bwd(y, dy, out=None):
    out = torch.empty_like(dy) if out is None else out
    _check(lib().xbar_relu_bwd(_dev(y), _dev(dy), _dev(out), y.numel(), _stream()))
    return out


def add(a, b, out=None):
    out = torch.empty_like(a) if out is None else out
    _check(lib().xbar_add(_dev(a), _dev(b), _dev(out), a.numel(), _stream()))
    return out


def sgd(p, g, lr):
    _check(lib().xbar_sgd(_dev(p), _dev(g), p.numel(), lr, _stream()))
    return p


def _bn_ws(rows, channels, ws, device):
    return _buffer(lib().xbar_bn_workspace_bytes(rows, channels), ws, device)


def bn_fwd(x, gamma, beta, eps=1e-5, ws=None):
    """xbar_bn_fwd on x[..., channels]: returns (y, mean, invstd)."""
    channels = x.shape[-1]
    rows = x.numel() // channels
    ws = _bn_ws(rows, channels, ws, x.device)
    y = torch.empty_like(x)
    mean = torch.empty(channels, dtype=torch.float32, device=x.device)
    invstd = torch.empty_like(mean)
    _check(lib().xbar_bn_fwd(_dev(x), _dev(gamma), _dev(beta), _dev(y), _dev(mean), _dev(invstd), rows, channels, eps,
                             C.c_void_p(ws.data_ptr()), ws.numel(), _stream()))
    return y, mean, invstd


def bn_bwd(x, dy, gamma, mean, invstd, ws=None):
    """xbar_bn_bwd: returns (dx, dgamma, dbeta)."""
    channels = x.shape[-1]
    rows = x.numel() // channels
    ws = _bn_ws(rows, channels, ws, x.device)
    dx = torch.empty_like(x)
    dgamma = torch.empty(channels, dtype=torch.float32, device=x.device)
    dbeta = torch.empty_like(dgamma)
    _check(lib().xbar_bn_bwd(_dev(x), _dev(dy), _dev(gamma), _dev(mean), _dev(invstd), _dev(dx), _dev(dgamma), _dev(dbeta),
                             rows, channels, C.c_void_p(ws.data_ptr()), ws.numel(), _stream()))
    return dx, dgamma, dbeta


def avgpool_fwd(x):
    """Global average pool of x[batch][h][w][channels] -> [batch][channels]."""
    b, ch = x.shape[0], x.shape[-1]
    y = torch.empty((b, ch), dtype=torch.float32, device=x.device)
    _check(lib().xbar_avgpool_fwd(_dev(x), _dev(y), b, x.numel() // (b * ch), ch, _stream()))
    return y


def avgpool_bwd(dy, shape):
    dx = torch.empty(shape, dtype=torch.float32, device=dy.device)
    b, ch = shape[0], shape[-1]
    _check(lib().xbar_avgpool_bwd(_dev(dy), _dev(dx), b, dx.numel() // (b * ch), ch, _stream()))
    return dx


def maxpool_fwd(x, geom):
    y = torch.empty((geom.batch, geom.out_h, geom.out_w, geom.in_c), dtype=torch.float32, device=x.device)
    arg = torch.empty(y.shape, dtype=torch.int32, device=x.device)
    _check(lib().xbar_maxpool_fwd(_dev(x), _dev(y), _dev(arg, torch.int32), C.byref(geom), _stream()))
    return y, arg


def maxpool_bwd(dy, arg, geom):
    dx = torch.empty((geom.batch, geom.in_h, geom.in_w, geom.in_c), dtype=torch.float32, device=dy.device)
    _check(lib().xbar_maxpool_bwd(_dev(dy), _dev(arg, torch.int32), _dev(dx), C.byref(geom), _stream()))
    return dx


def softmax_xent(logits, labels, scale):
    """xbar_softmax_xent: returns (per-sample loss, dlogits)."""
    b, classes = logits.shape
    loss = torch.empty(b, dtype=torch.float32, device=logits.device)
    dlogits = torch.empty_like(logits)
    _check(lib().xbar_softmax_xent(_dev(logits), _dev(labels, torch.int32), _dev(loss), _dev(dlogits), b, classes, scale,
                                   _stream()))
    return loss, dlogits


def shortcut_fwd(x, stride, out_channels):
    b, h, w, ch = x.shape
    y = torch.empty((b, (h + stride - 1) // stride, (w + stride - 1) // stride, out_channels), dtype=torch.float32,
                    device=x.device)
    _check(lib().xbar_shortcut_fwd(_dev(x), _dev(y), b, h, w, ch, stride, out_channels, _stream()))
    return y


def shortcut_bwd(dy, shape, stride):
    b, h, w, ch = shape
    dx = torch.empty(shape, dtype=torch.float32, device=dy.device)
    _check(lib().xbar_shortcut_bwd(_dev(dy), _dev(dx), b, h, w, ch, stride, dy.shape[-1], _stream()))
    return dx


def absmax(x, ws=None):
    """xbar_absmax: max |x| as a host float (synchronises: meant for calibration, not for the step)."""
    ws = _buffer(4096, ws, x.device)
    res = torch.empty(4, dtype=torch.float32, device=x.device)
    _check(lib().xbar_absmax(_dev(x), x.numel(), _dev(res), C.c_void_p(ws.data_ptr()), ws.numel(), _stream()))
    return float(res[0].item())


ADC_HIST_BINS = 4096


def conv_adc_histogram(cfg, planes, inp, geom, N, in_scale, op, bin_width, hist=None, ws=None):
    """xbar_conv_adc_histogram: as adc_histogram for a convolution layer (inp: the image for OP_FWD, the errors for
    OP_BWD)."""
    ws = _conv_ws(cfg, op, geom, N, ws, inp.device)
    if hist is None:
        hist = torch.zeros(ADC_HIST_BINS, dtype=torch.int64, device=inp.device)
    _check(lib().xbar_conv_adc_histogram(C.byref(cfg), C.c_void_p(planes.data_ptr()), _dev(inp), C.byref(geom), N, in_scale,
                                         op, bin_width, _dev(hist, torch.int64), C.c_void_p(ws.data_ptr()), ws.numel(),
                                         _stream()))
    return hist


def adc_histogram(cfg, planes, inp, K, N, in_scale, op, bin_width, hist=None, ws=None):
    """xbar_adc_histogram: adds the |column current| counts of this input to hist (int64[4096], device)."""
    M = inp.shape[0]
    ws = _buffer(workspace_bytes(cfg, op, M, K, N), ws, inp.device)
    if hist is None:
        hist = torch.zeros(ADC_HIST_BINS, dtype=torch.int64, device=inp.device)
    _check(lib().xbar_adc_histogram(C.byref(cfg), C.c_void_p(planes.data_ptr()), _dev(inp), M, K, N, in_scale, op,
                                    bin_width, _dev(hist, torch.int64), C.c_void_p(ws.data_ptr()), ws.numel(), _stream()))
    return hist
