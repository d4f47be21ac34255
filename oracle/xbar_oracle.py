"""TEST INFRASTRUCTURE: ctypes face of the scalar C oracle (oracle/xbar_oracle.c).

Argument marshalling only; all arithmetic of the method lives in the C file.  Nothing here is
imported by the product path.
"""
import ctypes as C
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from . import build as _build

INPUT_OFFSET = 1024
PULSE_CODED = 2048
PULSE_MAGNITUDE = 4096
VARIATION, WIRE_AAM, WIRE_PROFILE, UPD_NL, UPD_NOISE, DAC_LUT, INPUT_SIGNED, WIRE_AAM2, ADC_CURVE, ADC_PER_ARRAY = (
    1, 2, 4, 8, 16, 32, 64, 128, 256, 512)
STREAM_VARIATION, STREAM_WRITE = 1, 2


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


def make_config(**kw):
    """Config with the parameter values the paper states (Sec. V, Sec. VI-B); override by keyword."""
    c = Config()
    c.struct_size = C.sizeof(Config)
    c.abi_version = 2
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
    levels = (1 << c.stream_bits) - 1
    for i in range(16):
        c.dac_lut[i] = (lut[i] if lut is not None and i < len(lut) else (i / levels if i <= levels else 0.0))
    return c


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = C.CDLL(path)
        _lib.xo_normal.restype = C.c_double
        _lib.xo_normal.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint64]
        _lib.xo_quantize_weight.restype = C.c_int64
        _lib.xo_quantize_weight.argtypes = [C.c_float, C.c_float, C.c_int]
        _lib.xo_quantize_input.restype = C.c_int64
        _lib.xo_quantize_input.argtypes = [C.c_float, C.c_float, C.c_int, C.c_int]
        _lib.xo_quantize_input_offset.restype = C.c_int64
        _lib.xo_quantize_input_offset.argtypes = [C.c_float, C.c_float, C.c_int]
        _lib.xo_adc.restype = C.c_int64
        _lib.xo_adc.argtypes = [C.c_double, C.c_float, C.c_int]
        _lib.xo_adc_unsigned.restype = C.c_int64
        _lib.xo_adc_unsigned.argtypes = [C.c_double, C.c_float, C.c_int]
        _lib.xo_adc_curve.restype = C.c_int64
        _lib.xo_adc_curve.argtypes = [C.POINTER(C.c_float), C.c_double, C.c_float, C.c_int]
        assert _lib.xo_config_size() == C.sizeof(Config)
    return _lib


def _p(a, t):
    return None if a is None else a.ctypes.data_as(C.POINTER(t))


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _idx(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def n_slices(cfg):
    return cfg.weight_bits // cfg.slice_bits


def n_cycles(cfg):
    return cfg.input_bits // cfg.stream_bits


def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*ctr)
    k = (C.c_uint32 * 2)(*key)
    o = (C.c_uint32 * 4)()
    lib().xo_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def normal(seed, stream, step, i):
    return lib().xo_normal(seed, stream, step, i)


def normals(seed, stream, step, i0, count):
    f = lib().xo_normal
    return np.array([f(seed, stream, step, i0 + j) for j in range(count)])


def digits(mag, digit_bits, n_digits):
    d = (C.c_int32 * n_digits)()
    lib().xo_digits(C.c_uint64(mag), digit_bits, n_digits, d)
    return [int(x) for x in d]


def quantize_weight(w, w_max, bits):
    return int(lib().xo_quantize_weight(w, w_max, bits))


def quantize_input(x, x_scale, bits, is_signed):
    return int(lib().xo_quantize_input(x, x_scale, bits, int(is_signed)))


def quantize_input_offset(x, x_scale, bits):
    return int(lib().xo_quantize_input_offset(x, x_scale, bits))


def weight_sums(cfg, W, w_max):
    """(colsum[N], rowsum[K]) of the quantised weights: the digital correction of offset-binary inputs."""
    W = _f32(W)
    K, N = W.shape
    col, row = np.empty(N, dtype=np.int64), np.empty(K, dtype=np.int64)
    rc = lib().xo_weight_sums(C.byref(cfg), _p(W, C.c_float), K, N, C.c_float(w_max), _p(col, C.c_int64), _p(row, C.c_int64))
    assert rc == 0, rc
    return col, row


def adc(current, full_scale, bits):
    return int(lib().xo_adc(current, full_scale, bits))


def adc_unsigned(current, full_scale, bits):
    return int(lib().xo_adc_unsigned(C.c_double(current), C.c_float(full_scale), bits))


def adc_curve(curve, current, full_scale, bits):
    arr = (C.c_float * 17)(*curve)
    return int(lib().xo_adc_curve(arr, C.c_double(current), C.c_float(full_scale), bits))


def planes(cfg, W, w_max, step=0, profile=None, k_idx=None, n_idx=None, K_full=None, N_full=None):
    W = _f32(W)
    Ks, Ns = W.shape
    k_idx, n_idx = _idx(k_idx), _idx(n_idx)
    K_full = Ks if K_full is None else K_full
    N_full = Ns if N_full is None else N_full
    prof = None if profile is None else _f32(profile)
    # one converter per array: the arrays are kept apart, U[array][slice][k][n]
    shape = (2, n_slices(cfg), Ks, Ns) if cfg.flags & ADC_PER_ARRAY else (n_slices(cfg), Ks, Ns)
    U = np.empty(shape, dtype=np.float64)
    rc = lib().xo_planes(C.byref(cfg), _p(W, C.c_float), Ks, Ns, _p(k_idx, C.c_int32), _p(n_idx, C.c_int32),
                         K_full, N_full, C.c_float(w_max), C.c_uint64(step), _p(prof, C.c_float),
                         _p(U, C.c_double))
    assert rc == 0, rc
    return U


def device_conductances(cfg, W, w_max, step=0):
    """G[S][2][K][N]: conductance of every device before the wire model (array 0 = positive)."""
    W = _f32(W)
    K, N = W.shape
    G = np.zeros((n_slices(cfg), 2, K, N), dtype=np.float64)
    rc = lib().xo_device_conductances(C.byref(cfg), _p(W, C.c_float), K, N, C.c_float(w_max), C.c_uint64(step),
                                      _p(G, C.c_double))
    assert rc == 0, rc
    return G


def _tiles(cfg, length, transposed):
    t = cfg.xbar_cols if transposed else cfg.xbar_rows
    return (length + t - 1) // t


def fwd_planes(cfg, U, X, w_max, x_scale, want_codes=False, want_acc=False, wsum=None):
    """Forward VMM from generated planes U[S][K][Ns] ([2][S][K][Ns] with one converter per array);
    rows of X are independent.  Codes: [phase][cycle][slice][tile][m][n], with per-array converters
    [phase][cycle][slice][array][tile][m][n].  wsum: column sums of the quantised weights, needed
    with offset-binary signed inputs."""
    U = np.ascontiguousarray(U, dtype=np.float64)
    X = _f32(X)
    S, K, Ns = U.shape[-3:]
    M = X.shape[0]
    assert X.shape[1] == K and U.ndim == (4 if cfg.flags & ADC_PER_ARRAY else 3)
    Y = np.empty((M, Ns), dtype=np.float32)
    P = 2 if (cfg.flags & INPUT_SIGNED and not cfg.flags & INPUT_OFFSET) else 1
    arrays = (2,) if cfg.flags & ADC_PER_ARRAY else ()
    codes = np.empty((P, n_cycles(cfg), S) + arrays + (_tiles(cfg, K, False), M, Ns), dtype=np.int32) if want_codes else None
    acc = np.empty((M, Ns), dtype=np.int64) if want_acc else None
    wsum = None if wsum is None else np.ascontiguousarray(wsum, dtype=np.int64)
    assert wsum is None or wsum.shape == (Ns,)
    rc = lib().xo_fwd_planes(C.byref(cfg), _p(U, C.c_double), _p(X, C.c_float), _p(Y, C.c_float), M, K, Ns,
                             C.c_float(w_max), C.c_float(x_scale), _p(codes, C.c_int32), _p(acc, C.c_int64),
                             _p(wsum, C.c_int64))
    assert rc == 0, rc
    return _ret(Y, codes, acc)


def bwd_planes(cfg, U, dY, w_max, g_scale, want_codes=False, want_acc=False, wsum=None):
    """Backward VMM from generated planes U[S][Ks][N]; rows of dY are independent.  wsum: row sums of
    the quantised weights, needed with offset-binary signed inputs."""
    U = np.ascontiguousarray(U, dtype=np.float64)
    dY = _f32(dY)
    S, Ks, N = U.shape[-3:]
    M = dY.shape[0]
    assert dY.shape[1] == N and U.ndim == (4 if cfg.flags & ADC_PER_ARRAY else 3)
    dX = np.empty((M, Ks), dtype=np.float32)
    arrays = (2,) if cfg.flags & ADC_PER_ARRAY else ()
    P = 1 if cfg.flags & INPUT_OFFSET else 2
    codes = np.empty((P, n_cycles(cfg), S) + arrays + (_tiles(cfg, N, True), M, Ks), dtype=np.int32) if want_codes else None
    acc = np.empty((M, Ks), dtype=np.int64) if want_acc else None
    wsum = None if wsum is None else np.ascontiguousarray(wsum, dtype=np.int64)
    assert wsum is None or wsum.shape == (Ks,)
    rc = lib().xo_bwd_planes(C.byref(cfg), _p(U, C.c_double), _p(dY, C.c_float), _p(dX, C.c_float), M, Ks, N,
                             C.c_float(w_max), C.c_float(g_scale), _p(codes, C.c_int32), _p(acc, C.c_int64),
                             _p(wsum, C.c_int64))
    assert rc == 0, rc
    return _ret(dX, codes, acc)


def _ret(Y, codes, acc):
    out = [Y]
    if codes is not None:
        out.append(codes)
    if acc is not None:
        out.append(acc)
    return out[0] if len(out) == 1 else tuple(out)


def fwd(cfg, W, X, w_max, x_scale, step=0, profile=None, want_codes=False, want_acc=False):
    U = planes(cfg, W, w_max, step, profile)
    return fwd_planes(cfg, U, X, w_max, x_scale, want_codes, want_acc, weight_sums(cfg, W, w_max)[0])


def bwd(cfg, W, dY, w_max, g_scale, step=0, profile=None, want_codes=False, want_acc=False):
    U = planes(cfg, W, w_max, step, profile)
    return bwd_planes(cfg, U, dY, w_max, g_scale, want_codes, want_acc, weight_sums(cfg, W, w_max)[1])


def pulse_train(seed, stream, step, index, p, bl):
    f = lib().xo_pulse_train
    f.restype = C.c_uint32
    return int(f(C.c_uint64(seed), C.c_uint32(stream), C.c_uint64(step), C.c_uint64(index), C.c_double(p), C.c_int(bl)))


def pulse_code(p, bl, is_col):
    """Deterministic slot mask of a coded value (rows: whole frames, columns: sub-slots of every frame)."""
    f = lib().xo_pulse_code
    f.restype = C.c_uint32
    return int(f(C.c_double(p), C.c_int(bl), C.c_int(1 if is_col else 0)))


def pulse_frames(bl):
    tx, td = C.c_int(0), C.c_int(0)
    lib().xo_pulse_frames(C.c_int(bl), C.byref(tx), C.byref(td))
    return tx.value, td.value


def update_pulsed(cfg, W, X, dY, w_max, x_range, d_range, bl, dw_min, step=0, want_pulses=False, k_idx=None, n_idx=None,
                  K_full=None, N_full=None):
    """Pulse-level update, one sample at a time (stochastic trains, deterministic time codes with PULSE_CODED, or
    one pulse per sample whose height codes the value with PULSE_MAGNITUDE):
    returns the updated copy of W (and the signed number of pulses every device received, if asked).  With k_idx /
    n_idx the arguments are the devices at those rows / columns of a K_full x N_full layer."""
    W = _f32(W).copy()
    X, dY = _f32(X), _f32(dY)
    M, K = X.shape
    N = dY.shape[1]
    assert W.shape == (K, N) and dY.shape[0] == M
    pulses = np.empty((K, N), dtype=np.int64) if want_pulses else None
    k_idx, n_idx = _idx(k_idx), _idx(n_idx)
    assert (k_idx is None or len(k_idx) == K) and (n_idx is None or len(n_idx) == N)
    rc = lib().xo_update_pulsed_at(C.byref(cfg), _p(W, C.c_float), _p(X, C.c_float), _p(dY, C.c_float), M, K, N,
                                   _p(k_idx, C.c_int32), _p(n_idx, C.c_int32), K if K_full is None else K_full,
                                   N if N_full is None else N_full, C.c_float(w_max), C.c_float(x_range),
                                   C.c_float(d_range), C.c_int(bl), C.c_float(dw_min), C.c_uint64(step),
                                   _p(pulses, C.c_int64))
    assert rc == 0, rc
    return (W, pulses) if want_pulses else W


def update(cfg, W, X, dY, w_max, grad_scale, lr, step=0, k_idx=None, n_idx=None, N_full=None, want_grad=False):
    """Returns the updated copy of W (and the raw gradient sum if asked)."""
    W = _f32(W).copy()
    X, dY = _f32(X), _f32(dY)
    Ks, Ns = W.shape
    M = X.shape[0]
    assert X.shape == (M, Ks) and dY.shape == (M, Ns)
    k_idx, n_idx = _idx(k_idx), _idx(n_idx)
    N_full = Ns if N_full is None else N_full
    grad = np.empty((Ks, Ns), dtype=np.float64) if want_grad else None
    rc = lib().xo_update(C.byref(cfg), _p(W, C.c_float), _p(X, C.c_float), _p(dY, C.c_float), M, Ks, Ns,
                         _p(k_idx, C.c_int32), _p(n_idx, C.c_int32), N_full, C.c_float(w_max),
                         C.c_float(grad_scale), C.c_float(lr), C.c_uint64(step), _p(grad, C.c_double))
    assert rc == 0
    return (W, grad) if want_grad else W


def pair_init(W, w_max):
    """Positive / negative device states of a weight matrix, placed symmetrically about mid-range."""
    W = _f32(W)
    Gp, Gn = np.empty_like(W), np.empty_like(W)
    lib().xo_pair_init(_p(W, C.c_float), _p(Gp, C.c_float), _p(Gn, C.c_float), C.c_size_t(W.size), C.c_float(w_max))
    return Gp, Gn


def update_pair(cfg, Gp, Gn, X, dY, w_max, grad_scale, lr, step=0):
    """Update with per-polarity device state: returns the updated copies (Gp, Gn, W = w_max (Gp - Gn))."""
    Gp, Gn = _f32(Gp).copy(), _f32(Gn).copy()
    X, dY = _f32(X), _f32(dY)
    K, N = Gp.shape
    M = X.shape[0]
    assert Gn.shape == (K, N) and X.shape == (M, K) and dY.shape == (M, N)
    W = np.empty((K, N), dtype=np.float32)
    rc = lib().xo_update_pair(C.byref(cfg), _p(Gp, C.c_float), _p(Gn, C.c_float), _p(W, C.c_float), _p(X, C.c_float),
                              _p(dY, C.c_float), M, K, N, C.c_float(w_max), C.c_float(grad_scale), C.c_float(lr),
                              C.c_uint64(step))
    assert rc == 0
    return Gp, Gn, W


def rows_parallel(fn, U, X, threads):
    """Runs fn(U, X_block) over disjoint row blocks on `threads` host threads (the C code is
    re-entrant and ctypes drops the GIL).  Returns the stacked outputs."""
    M = X.shape[0]
    threads = max(1, min(threads, M))
    bounds = np.linspace(0, M, threads + 1).astype(int)
    blocks = [(bounds[i], bounds[i + 1]) for i in range(threads) if bounds[i + 1] > bounds[i]]
    with ThreadPoolExecutor(max_workers=len(blocks)) as ex:
        outs = list(ex.map(lambda b: fn(U, X[b[0]:b[1]]), blocks))
    return np.concatenate(outs, axis=0)
