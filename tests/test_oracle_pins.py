"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Each test checks the oracle against something other than itself: a published known-answer vector, a
closed form, a textbook special case (integer matmul, plain SGD, series resistors), the exact circuit
solution of a small tile, statistics of the random draws, or a brute-force re-derivation on tiny
inputs.  The paper prints no numeric worked example, so there are no paper-value fixtures.
"""
import math
import os

import numpy as np
import pytest
from scipy import stats

import workloads
from oracle import nodal

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


# ------------------------------------------------------------------------------------------------
# random numbers
# ------------------------------------------------------------------------------------------------
def test_philox_known_answers(xo):
    n = 0
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(t, 16) for t in line.split()]
        assert xo.philox4x32_10(w[0:4], w[4:6]) == w[6:10]
        n += 1
    assert n == 2


def test_normal_moments_and_distribution(xo):
    z = xo.normals(seed=7, stream=xo.STREAM_WRITE, step=3, i0=0, count=200000)
    assert abs(z.mean()) < 4 / math.sqrt(z.size)
    assert abs(z.var() - 1.0) < 0.02
    assert abs(stats.skew(z)) < 0.03 and abs(stats.kurtosis(z)) < 0.06
    assert stats.kstest(z, "norm").pvalue > 1e-3
    # the four numbers of one block and neighbouring blocks are uncorrelated
    for lag in (1, 2, 3, 4):
        assert abs(np.corrcoef(z[:-lag], z[lag:])[0, 1]) < 0.01


def test_normal_keying(xo):
    a = xo.normals(1, 1, 0, 0, 64)
    assert np.array_equal(a, xo.normals(1, 1, 0, 0, 64))          # reproducible
    for other in (xo.normals(2, 1, 0, 0, 64), xo.normals(1, 2, 0, 0, 64), xo.normals(1, 1, 1, 0, 64),
                  xo.normals(1 + (1 << 32), 1, 0, 0, 64), xo.normals(1, 1, 1 << 32, 0, 64),
                  xo.normals(1, 1, 0, 1 << 34, 64)):
        assert not np.any(a == other)                            # every key part matters


# ------------------------------------------------------------------------------------------------
# encodings
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("digit_bits,n_digits", [(2, 8), (1, 16), (4, 4), (2, 4), (4, 2), (1, 8)])
def test_digit_recombination_is_identity(xo, digit_bits, n_digits):
    top = 1 << (digit_bits * n_digits)
    values = range(top) if top <= 65536 else range(0, top, 7)
    for v in values:
        d = xo.digits(v, digit_bits, n_digits)
        assert all(0 <= x < (1 << digit_bits) for x in d)
        assert sum(x << (digit_bits * s) for s, x in enumerate(d)) == v


def test_weight_quantiser_grid_ties_clamp(xo):
    for bits in (8, 16):
        qw = (1 << bits) - 1
        for j in (-qw, -3, -1, 0, 1, 2, 77, qw):               # grid points map to themselves
            assert xo.quantize_weight(np.float32(j / qw * 0.5), 0.5, bits) == j
    # exact ties round to even: w/w_max * 255 = 0.5, 1.5, 2.5 with w_max = 255
    assert [xo.quantize_weight(x, 255.0, 8) for x in (0.5, 1.5, 2.5, -0.5, -1.5)] == [0, 2, 2, 0, -2]
    assert xo.quantize_weight(9.0, 1.0, 8) == 255 and xo.quantize_weight(-9.0, 1.0, 8) == -255


def test_input_quantiser(xo):
    assert [xo.quantize_input(x, 255.0, 8, True) for x in (0.5, 1.5, -2.5, 300.0, -300.0)] == [0, 2, -2, 255, -255]
    assert [xo.quantize_input(x, 255.0, 8, False) for x in (-7.0, 3.0, 300.0)] == [0, 3, 255]
    assert xo.quantize_input(1.0, 1.0, 4, False) == 15


def test_adc_closed_form(xo):
    # lsb = 2: odd currents sit exactly between two codes -> even code; saturation at +-Q
    q = 127
    for cur, code in ((0, 0), (1, 0), (2, 1), (3, 2), (5, 2), (7, 4), (-3, -2), (253, 126), (254, 127),
                      (255, 127), (1000, 127), (-255, -127), (-1e9, -127)):
        assert xo.adc(float(cur), 2.0 * q, 8) == code
    # lsb = 128/127: current 64 is an exact tie between 63 and 64
    assert xo.adc(64.0, 128.0, 8) == 64 and xo.adc(192.0, 128.0, 8) == 127
    # ramp across the clip point, lsb = 1
    for bits in (4, 6, 8, 12):
        q = (1 << (bits - 1)) - 1
        for cur in range(-q - 5, q + 6):
            assert xo.adc(float(cur), float(q), bits) == max(-q, min(q, cur))
        assert xo.adc(0.49, float(q), bits) == 0 and xo.adc(0.51, float(q), bits) == 1


# ------------------------------------------------------------------------------------------------
# ideal crossbars: exact integer arithmetic
# ------------------------------------------------------------------------------------------------
def _ideal_cfg(xo, R, C, stream_bits, slice_bits, weight_bits, signed, adc_bits=None):
    worst = max(R, C) * ((1 << stream_bits) - 1) * ((1 << slice_bits) - 1)
    adc_bits = adc_bits or (int(math.ceil(math.log2(worst + 1))) + 1)
    q = (1 << (adc_bits - 1)) - 1
    return xo.make_config(xbar_rows=R, xbar_cols=C, weight_bits=weight_bits, slice_bits=slice_bits,
                          input_bits=8, stream_bits=stream_bits, adc_bits=adc_bits,
                          flags=xo.INPUT_SIGNED if signed else 0, adc_fs_fwd=float(q), adc_fs_bwd=float(q))


def _int_grid_tensors(rng, M, K, N, wbits, signed):
    """Tensors that sit exactly on the quantiser grids, so the integers are known without quantising."""
    qw, qa = (1 << wbits) - 1, 255
    q = rng.integers(-qw, qw + 1, size=(K, N))
    a = rng.integers(-qa if signed else 0, qa + 1, size=(M, K))
    w_max, x_scale = 1.0, 1.0
    W = (q.astype(np.float64) / qw).astype(np.float32)
    X = (a.astype(np.float64) / qa).astype(np.float32)
    return q, a, W, X, w_max, x_scale


def test_one_converter_per_array(xo):
    """Variant: every array has an unsigned converter of its own, the codes are subtracted digitally."""
    rng = np.random.default_rng(12)
    # converter closed form: all 2^bits - 1 codes on one side, nothing below zero
    for bits, fs in ((8, 64.0), (4, 10.0)):
        q = (1 << bits) - 1
        assert xo.adc_unsigned(-3.0, fs, bits) == 0 and xo.adc_unsigned(2 * fs, fs, bits) == q
        for cur in rng.uniform(0, fs, size=200):
            assert xo.adc_unsigned(cur, fs, bits) == int(np.rint(cur * float(np.float32(q) / np.float32(fs))))
    K, N, M = 20, 9, 6
    q_w = rng.integers(-15, 16, size=(K, N))
    W = (q_w / 15.0).astype(np.float32)
    X = (rng.integers(-255, 256, size=(M, K)) / 255.0).astype(np.float32)
    kw = dict(xbar_rows=8, xbar_cols=8, weight_bits=4, slice_bits=2, input_bits=8, stream_bits=4, r_min=1e4, r_max=1e5)
    # planes: each array on its own, their difference is the merged plane of the one-converter model
    merged = xo.planes(xo.make_config(flags=xo.WIRE_AAM, **kw), W, 1.0)
    apart = xo.planes(xo.make_config(flags=xo.WIRE_AAM | xo.ADC_PER_ARRAY, **kw), W, 1.0)
    assert apart.shape == (2,) + merged.shape and (apart > 0).all()
    assert np.allclose(apart[0] - apart[1], merged, rtol=0, atol=1e-12)
    # ideal arrays: the resting conductance of the other array is still there (Gmin / dG = 1/3 here)
    ideal = xo.planes(xo.make_config(flags=xo.ADC_PER_ARRAY, **kw), W, 1.0)
    dig = (np.abs(q_w) & 3)
    assert np.allclose(ideal[0, 0], 1.0 / 3.0 + np.where(q_w > 0, dig, 0), atol=1e-12)
    assert np.allclose(ideal[1, 0], 1.0 / 3.0 + np.where(q_w < 0, dig, 0), atol=1e-12)
    # brute force of one output through both converters, codes and sum
    cfg = xo.make_config(flags=xo.ADC_PER_ARRAY | xo.INPUT_SIGNED, adc_bits=6, adc_fs_fwd=40.0, **kw)
    Y, codes, acc = xo.fwd(cfg, W, X, 1.0, 1.0, want_codes=True, want_acc=True)
    assert codes.shape == (2, 2, 2, 2, 3, M, N) and codes.min() >= 0 and codes.max() <= 63
    a = np.rint(X.astype(np.float64) * 255).astype(int)
    m, n = 3, 5
    total = 0
    for p in range(2):
        mag = np.where(a[m] > 0, a[m], 0) if p == 0 else np.where(a[m] < 0, -a[m], 0)
        for b in range(2):
            digit = (mag >> (4 * b)) & 15
            for s in range(2):
                for pol in range(2):
                    for t in range(3):
                        rows = slice(8 * t, min(8 * t + 8, K))
                        cur = float((digit[rows] * ideal[pol, s, rows, n]).sum())
                        code = min(max(int(np.rint(cur * float(np.float32(63) / np.float32(40.0)))), 0), 63)
                        assert codes[p, b, s, pol, t, m, n] == code
                        total += (1 if p == 0 else -1) * (1 if pol == 0 else -1) * code * (1 << (2 * s + 4 * b))
    assert acc[m, n] == total
    assert abs(Y[m, n] - total * (40.0 / 63) / (255 * 15)) < 1e-6
    # with a fine converter the result approaches the one-converter model (the resting currents cancel)
    fine1 = xo.fwd(xo.make_config(flags=xo.INPUT_SIGNED, adc_bits=16, adc_fs_fwd=400.0, **kw), W, X, 1.0, 1.0)
    fine2 = xo.fwd(xo.make_config(flags=xo.INPUT_SIGNED | xo.ADC_PER_ARRAY, adc_bits=16, adc_fs_fwd=400.0, **kw), W, X, 1.0, 1.0)
    assert np.abs(fine1 - fine2).max() < 2e-3 * np.abs(fine1).max()


def test_offset_binary_signed_inputs(xo):
    """Variant: signed inputs streamed in one phase as offset-binary codes, half-range removed digitally."""
    rng = np.random.default_rng(21)
    # the code: ends of the range, the middle (half a step off, to the even code), clamping, monotone,
    # coded value within half a step (one step = 2 scale / Qa) of the input
    for bits in (8, 4, 3):
        qa = (1 << bits) - 1
        assert xo.quantize_input_offset(-2.0, 2.0, bits) == 0 and xo.quantize_input_offset(2.0, 2.0, bits) == qa
        assert xo.quantize_input_offset(-9.0, 2.0, bits) == 0 and xo.quantize_input_offset(9.0, 2.0, bits) == qa
        assert xo.quantize_input_offset(0.0, 2.0, bits) == 2 * int(np.rint((qa / 2.0) / 2.0))       # 128, 8, 4
        xs = np.sort(rng.uniform(-2, 2, size=300)).astype(np.float32)
        us = [xo.quantize_input_offset(float(x), 2.0, bits) for x in xs]
        assert all(b >= a for a, b in zip(us, us[1:]))
        coded = (2.0 * np.array(us) - qa) / qa * 2.0
        assert np.abs(coded - xs).max() <= 2.0 / qa + 1e-6
    K, N, M = 21, 10, 7
    q_w = rng.integers(-15, 16, size=(K, N))
    W = (q_w / 15.0).astype(np.float32)
    X = rng.uniform(-1, 1, size=(M, K)).astype(np.float32)
    dY = rng.uniform(-1, 1, size=(M, N)).astype(np.float32)
    kw = dict(xbar_rows=8, xbar_cols=8, weight_bits=4, slice_bits=2, input_bits=8, stream_bits=4, r_min=1e4, r_max=1e5)
    # weight sums against numpy on the known integers
    col, row = xo.weight_sums(xo.make_config(**kw), W, 1.0)
    assert np.array_equal(col, q_w.sum(axis=0)) and np.array_equal(row, q_w.sum(axis=1))
    # ideal arrays, lossless converters: the product of the coded inputs and the quantised weights, exactly
    lossless = dict(adc_bits=16, adc_fs_fwd=32767.0, adc_fs_bwd=32767.0)
    cfg = xo.make_config(flags=xo.INPUT_SIGNED | xo.INPUT_OFFSET, **kw, **lossless)
    u = np.array([[xo.quantize_input_offset(float(x), 1.0, 8) for x in r] for r in X])
    Y, codes, acc = xo.fwd(cfg, W, X, 1.0, 1.0, want_codes=True, want_acc=True)
    assert codes.shape == (1, 2, 2, 3, M, N)                                   # one phase
    assert np.array_equal(acc, u @ q_w)
    want = ((2 * u - 255) @ q_w) / (255.0 * 15.0)
    assert np.abs(Y - want).max() <= 1e-6 * np.abs(want).max()
    ud = np.array([[xo.quantize_input_offset(float(x), 1.0, 8) for x in r] for r in dY])
    dX, codes_b = xo.bwd(cfg, W, dY, 1.0, 1.0, want_codes=True)
    assert codes_b.shape == (1, 2, 2, 2, M, K)
    want_b = ((2 * ud - 255) @ q_w.T) / (255.0 * 15.0)
    assert np.abs(dX - want_b).max() <= 1e-6 * np.abs(want_b).max()
    # against the two-phase scheme: the inputs differ by the two quantisation errors (half of 2/Qa and of 1/Qa)
    two = xo.fwd(xo.make_config(flags=xo.INPUT_SIGNED, **kw, **lossless), W, X, 1.0, 1.0)
    bound = 1.5 / 255.0 * np.abs(q_w / 15.0).sum(axis=0)
    assert (np.abs(Y - two) <= bound + 1e-6).all() and np.abs(Y - two).max() > 0
    # without the sign flag the forward inputs are unsigned and the scheme does not apply
    Xp = np.abs(X)
    assert np.array_equal(xo.fwd(xo.make_config(flags=xo.INPUT_OFFSET, **kw, **lossless), W, Xp, 1.0, 1.0),
                          xo.fwd(xo.make_config(**kw, **lossless), W, Xp, 1.0, 1.0))
    # brute force of one output with non-ideal arrays and coarse converters (differential, then one per array)
    for extra, q_adc in ((0, 31), (xo.ADC_PER_ARRAY, 63)):
        cfg = xo.make_config(flags=xo.INPUT_SIGNED | xo.INPUT_OFFSET | xo.WIRE_AAM | extra, adc_bits=6, adc_fs_fwd=50.0, **kw)
        U = xo.planes(cfg, W, 1.0)
        Y, codes, acc = xo.fwd(cfg, W, X, 1.0, 1.0, want_codes=True, want_acc=True)
        gain = float(np.float32(q_adc) / np.float32(50.0))
        m, n = 4, 6
        total = 0
        for b in range(2):
            digit = (u[m] >> (4 * b)) & 15
            for s in range(2):
                for pol in range(2 if extra else 1):
                    for t in range(3):
                        rows = slice(8 * t, min(8 * t + 8, K))
                        plane = U[pol, s] if extra else U[s]
                        cur = float((digit[rows] * plane[rows, n]).sum())
                        code = int(np.rint(cur * gain))
                        code = min(max(code, 0 if extra else -q_adc), q_adc)
                        got = codes[0, b, s, pol, t, m, n] if extra else codes[0, b, s, t, m, n]
                        assert got == code
                        total += (-1 if pol else 1) * code * (1 << (2 * s + 4 * b))
        assert acc[m, n] == total
        want = (2.0 * total * (50.0 / q_adc) - 255.0 * q_w[:, n].sum()) / (255.0 * 15.0)
        assert abs(Y[m, n] - want) < 1e-6
    # the correction needs the weight sums
    with pytest.raises(AssertionError):
        xo.fwd_planes(cfg, U, X, 1.0, 1.0)


def test_adc_transfer_curve(xo):
    identity = [-1.0 + i / 8.0 for i in range(17)]
    rng = np.random.default_rng(6)
    for bits, fs in ((8, 64.0), (6, 100.0), (12, 3.0)):
        q = (1 << (bits - 1)) - 1
        for cur in rng.uniform(-1.5 * fs, 1.5 * fs, size=400):
            assert xo.adc_curve(identity, cur, fs, bits) == xo.adc(cur, fs, bits)
        # a curve that is linear with slope 1/2: half the code, full range never reached
        half = [0.5 * v for v in identity]
        for cur in rng.uniform(-fs, fs, size=200):
            want = int(np.rint(0.5 * cur * float(np.float32(q) / np.float32(fs))))
            assert abs(xo.adc_curve(half, cur, fs, bits) - want) <= 1          # rne of a halved value: ties may differ
        assert xo.adc_curve(half, 10 * fs, fs, bits) == int(np.rint(0.5 * q))
        # compressive curve: monotone in the current, equal to the knot values at the knots, saturating
        bowed = [float(np.tanh(1.5 * v) / np.tanh(1.5)) for v in identity]
        codes = [xo.adc_curve(bowed, cur, fs, bits) for cur in np.linspace(-1.2 * fs, 1.2 * fs, 301)]
        assert all(b >= a for a, b in zip(codes, codes[1:])) and codes[0] == -q and codes[-1] == q
        for i, v in enumerate(identity):
            gain = float(np.float32(q) / np.float32(fs))
            assert abs(xo.adc_curve(bowed, v * q / gain, fs, bits) - q * bowed[i]) <= 0.5 + 1e-9
    # the curve is used by the layer: a compressive converter changes the outputs, the identity curve does not
    W = rng.uniform(-1, 1, size=(40, 12)).astype(np.float32)
    X = rng.uniform(0, 1, size=(5, 40)).astype(np.float32)
    base = xo.make_config(xbar_rows=16, xbar_cols=16, adc_bits=6, adc_fs_fwd=8.0)
    same = xo.make_config(xbar_rows=16, xbar_cols=16, adc_bits=6, adc_fs_fwd=8.0, flags=xo.ADC_CURVE)
    bent = xo.make_config(xbar_rows=16, xbar_cols=16, adc_bits=6, adc_fs_fwd=8.0, flags=xo.ADC_CURVE, adc_curve=bowed)
    assert np.array_equal(xo.fwd(base, W, X, 1.0, 1.0), xo.fwd(same, W, X, 1.0, 1.0))
    assert not np.array_equal(xo.fwd(base, W, X, 1.0, 1.0), xo.fwd(bent, W, X, 1.0, 1.0))


@pytest.mark.parametrize("R,C,sb,slb,wb,signed,M,K,N", [
    (8, 8, 1, 2, 8, False, 5, 19, 11),
    (8, 4, 4, 2, 8, True, 3, 8, 9),
    (16, 16, 2, 1, 8, True, 4, 40, 17),
    (64, 64, 4, 2, 8, True, 6, 150, 70),
    (128, 128, 1, 2, 16, False, 3, 147, 64),
])
def test_fwd_ideal_full_precision_is_integer_matmul(xo, R, C, sb, slb, wb, signed, M, K, N):
    rng = np.random.default_rng(R + K)
    cfg = _ideal_cfg(xo, R, C, sb, slb, wb, signed)
    q, a, W, X, w_max, x_scale = _int_grid_tensors(rng, M, K, N, wb, signed)
    Y, acc = xo.fwd(cfg, W, X, w_max, x_scale, want_acc=True)
    assert np.array_equal(acc, a @ q)                              # textbook integer matmul
    ref = (a @ q).astype(np.float64) / (255.0 * ((1 << wb) - 1))
    assert np.allclose(Y, ref, rtol=1e-6, atol=0)


@pytest.mark.parametrize("R,C,sb,slb,wb,M,K,N", [(8, 4, 1, 2, 8, 5, 19, 11), (64, 64, 4, 2, 8, 4, 70, 150),
                                                (16, 32, 2, 2, 16, 3, 33, 65)])
def test_bwd_ideal_full_precision_is_transposed_integer_matmul(xo, R, C, sb, slb, wb, M, K, N):
    rng = np.random.default_rng(C + N)
    cfg = _ideal_cfg(xo, R, C, sb, slb, wb, True)
    q, _, W, _, w_max, _ = _int_grid_tensors(rng, M, K, N, wb, True)
    e = rng.integers(-255, 256, size=(M, N))
    dY = (e.astype(np.float64) / 255 * 0.01).astype(np.float32)
    dX, acc = xo.bwd(cfg, W, dY, w_max, 0.01, want_acc=True)
    assert np.array_equal(acc, e @ q.T)
    assert np.allclose(dX, (e @ q.T) * (0.01 / (255.0 * ((1 << wb) - 1))), rtol=1e-6, atol=0)


def test_fwd_ideal_adc_code_closed_form(xo):
    # all rows driven with the same digit a, all devices of a column hold the same digit d:
    # tile current = rows_in_tile * a * d exactly, code = clamp(rne(I / lsb))
    R, K, N, M = 16, 40, 4, 1
    cfg = xo.make_config(xbar_rows=R, xbar_cols=R, weight_bits=2, slice_bits=2, input_bits=4, stream_bits=4,
                         adc_bits=6, adc_fs_fwd=62.0, adc_fs_bwd=62.0)     # Q = 31, lsb = 2
    for a in (1, 5, 15):
        for d in (-3, -1, 0, 2, 3):
            W = np.full((K, N), d / 3.0, dtype=np.float32)
            X = np.full((M, K), a / 15.0, dtype=np.float32)
            Y, codes, acc = xo.fwd(cfg, W, X, 1.0, 1.0, want_codes=True, want_acc=True)
            rows = [16, 16, 8]                                       # ragged last tile has 8 rows
            expect = []
            for r in rows:
                cur = r * a * d
                half = cur / 2.0
                c = math.floor(half) if half - math.floor(half) < 0.5 else math.ceil(half)
                if half - math.floor(half) == 0.5:
                    c = math.floor(half) if math.floor(half) % 2 == 0 else math.ceil(half)
                expect.append(max(-31, min(31, c)))
            assert codes.shape == (1, 1, 1, 3, M, N)
            assert [int(codes[0, 0, 0, t, 0, 0]) for t in range(3)] == expect
            assert int(acc[0, 0]) == sum(expect)
            assert Y[0, 0] == np.float32(sum(expect) * 2.0 / (15 * 3))


def test_fwd_ideal_monotone_in_adc_bits(xo):
    rng = np.random.default_rng(5)
    g = workloads.Gemm("t", 96, 40, 6, False, 1)
    W, X, _ = workloads.layer_tensors_np(g, 11)
    w_max, x_scale = float(np.abs(W).max()), float(X.max())
    errs = []
    for bits in (4, 6, 8, 10, 14):
        q = (1 << (bits - 1)) - 1
        cfg = xo.make_config(xbar_rows=32, xbar_cols=32, weight_bits=8, slice_bits=2, input_bits=8, stream_bits=4,
                             adc_bits=bits, adc_fs_fwd=32.0 * 15 * 3, adc_fs_bwd=32.0 * 15 * 3)
        Y = xo.fwd(cfg, W, X, w_max, x_scale)
        errs.append(np.linalg.norm(Y - X.astype(np.float64) @ W.astype(np.float64)))
    assert all(errs[i + 1] <= errs[i] * 1.05 for i in range(len(errs) - 1)) and errs[-1] < 0.05 * errs[0]


# ------------------------------------------------------------------------------------------------
# non-ideal arrays
# ------------------------------------------------------------------------------------------------
def _device_g(cfg, d):
    g_min, g_max = 1.0 / cfg.r_max, 1.0 / cfg.r_min
    return g_min + d * (g_max - g_min) / ((1 << cfg.slice_bits) - 1)


def test_aam_single_cell_is_series_resistors(xo):
    cfg = xo.make_config(xbar_rows=1, xbar_cols=1, weight_bits=2, slice_bits=2, flags=xo.WIRE_AAM,
                         r_row=30.0, r_col=500.0, r_source=1e3, r_sense=2e3, r_min=1e4, r_max=1e5)
    dg = (1 / 1e4 - 1 / 1e5) / 3
    for d in (1, 2, 3):
        U = xo.planes(cfg, np.array([[d / 3.0]], dtype=np.float32), 1.0)
        series = lambda g: 1.0 / (1.0 / g + 1e3 + 30.0 + 500.0 + 2e3)
        expect = (series(_device_g(cfg, d)) - series(_device_g(cfg, 0))) / dg
        assert abs(U[0, 0, 0] - expect) < 1e-12 * abs(expect)
        Un = xo.planes(cfg, np.array([[-d / 3.0]], dtype=np.float32), 1.0)
        assert Un[0, 0, 0] == -U[0, 0, 0]
        # and the exact circuit solution of a single cell is that same series connection
        E = nodal.effective_conductance([[_device_g(cfg, d)]], 30.0, 500.0, 1e3, 2e3)
        assert abs(E[0, 0] - series(_device_g(cfg, d))) < 1e-12 * E[0, 0]


def test_aam_without_wire_resistance_is_ideal(xo):
    rng = np.random.default_rng(2)
    W = rng.uniform(-1, 1, size=(20, 12)).astype(np.float32)
    ideal = xo.make_config(xbar_rows=8, xbar_cols=8)
    aam0 = xo.make_config(xbar_rows=8, xbar_cols=8, flags=xo.WIRE_AAM, r_row=0.0, r_col=0.0)
    assert np.allclose(xo.planes(aam0, W, 1.0), xo.planes(ideal, W, 1.0), rtol=0, atol=1e-12)


def test_aam_geometry_against_path_enumeration(xo):
    # plane value of device (i, j) inside every tile, re-derived by walking the path cell by cell
    R, C, K, N = 4, 3, 10, 7
    cfg = xo.make_config(xbar_rows=R, xbar_cols=C, weight_bits=4, slice_bits=2, flags=xo.WIRE_AAM,
                         r_row=2.0, r_col=7.0, r_source=11.0, r_sense=13.0, r_min=1e3, r_max=1e4)
    rng = np.random.default_rng(3)
    qv = rng.integers(-15, 16, size=(K, N))
    U = xo.planes(cfg, (qv / 15.0).astype(np.float32), 1.0)
    dg = (1e-3 - 1e-4) / 3
    for k in range(K):
        for n in range(N):
            i, j = k % R, n % C
            path = 11.0 + 13.0
            for _ in range(j + 1):          # row-wire cells from the driver up to and including column j
                path += 2.0
            for _ in range(i, R):           # column-wire cells from row i down to the sense end
                path += 7.0
            for s in range(2):
                d = (abs(int(qv[k, n])) >> (2 * s)) & 3
                on = 1.0 / (1.0 / _device_g(cfg, d) + path)
                off = 1.0 / (1.0 / _device_g(cfg, 0) + path)
                expect = math.copysign(1.0, qv[k, n]) * (on - off) / dg if qv[k, n] else 0.0
                assert abs(U[s, k, n] - expect) < 1e-12


@pytest.mark.parametrize("R,C", [(2, 2), (4, 4), (8, 8), (8, 3)])
def test_aam_converges_to_exact_circuit_for_high_device_resistance(xo, R, C):
    # Sec. IV-D: negligible error when the device resistance range is far above the wire
    # resistance, considerable error when it is low.
    rng = np.random.default_rng(R * 10 + C)
    d = rng.integers(0, 4, size=(R, C))
    errs = []
    for r_min in (1e3, 1e4, 1e5, 1e6):
        cfg = xo.make_config(xbar_rows=R, xbar_cols=C, weight_bits=2, slice_bits=2, flags=xo.WIRE_AAM,
                             r_min=r_min, r_max=10 * r_min, r_row=1.0, r_col=4.6)
        dg = (1 / r_min - 0.1 / r_min) / 3
        U = xo.planes(cfg, (d / 3.0).astype(np.float32), 1.0)[0]
        G = _device_g(cfg, d.astype(np.float64))
        E_on = nodal.effective_conductance(G, 1.0, 4.6)
        E_off = nodal.effective_conductance(np.full((R, C), _device_g(cfg, 0)), 1.0, 4.6)
        exact = (E_on - E_off) / dg
        errs.append(np.abs(U - exact).max())
    assert all(errs[i + 1] < errs[i] * 0.2 for i in range(3))
    assert errs[-1] < 1e-3 * R * C / 64 + 1e-5


def _exact_plane(cfg, d, rows=None, cols=None, scale=1.0):
    """(E+ - E-) / dG of the exact circuit for non-negative digits d on one tile (absent devices: G = 0)."""
    R, C = cfg.xbar_rows, cfg.xbar_cols
    Gp = np.zeros((R, C))
    Gn = np.zeros((R, C))
    rows, cols = rows or R, cols or C
    Gp[:rows, :cols] = _device_g(cfg, d.astype(np.float64))
    Gn[:rows, :cols] = _device_g(cfg, 0)
    dg = _device_g(cfg, 1) - _device_g(cfg, 0)
    wires = (cfg.r_row * scale, cfg.r_col * scale, cfg.r_source * scale, cfg.r_sense * scale)
    E = nodal.effective_conductance(Gp, *wires) - nodal.effective_conductance(Gn, *wires)
    return (E / dg)[:rows, :cols]


def test_aam2_single_cell_and_isolated_devices_equal_single_path_model(xo):
    kw = dict(weight_bits=2, slice_bits=2, r_row=30.0, r_col=500.0, r_source=1e3, r_sense=2e3, r_min=1e4)
    for d in (1, 2, 3):
        W = np.array([[d / 3.0]], dtype=np.float32)
        one = xo.planes(xo.make_config(xbar_rows=1, xbar_cols=1, r_max=1e5, flags=xo.WIRE_AAM, **kw), W, 1.0)
        two = xo.planes(xo.make_config(xbar_rows=1, xbar_cols=1, r_max=1e5, flags=xo.WIRE_AAM2, **kw), W, 1.0)
        assert abs(one[0, 0, 0] - two[0, 0, 0]) < 1e-12
    # one conducting device per row and per column (the others practically open): nothing is shared
    R = 6
    perm = np.random.default_rng(5).permutation(R)
    W = np.zeros((R, R), dtype=np.float32)
    W[np.arange(R), perm] = 1.0
    one = xo.planes(xo.make_config(xbar_rows=R, xbar_cols=R, r_max=1e16, flags=xo.WIRE_AAM, **kw), W, 1.0)
    two = xo.planes(xo.make_config(xbar_rows=R, xbar_cols=R, r_max=1e16, flags=xo.WIRE_AAM2, **kw), W, 1.0)
    assert np.abs(one - two).max() < 1e-9 and np.abs(two).max() > 0.5


def test_aam2_without_wire_resistance_is_ideal(xo):
    rng = np.random.default_rng(2)
    W = rng.uniform(-1, 1, size=(20, 12)).astype(np.float32)
    ideal = xo.make_config(xbar_rows=8, xbar_cols=8)
    aam0 = xo.make_config(xbar_rows=8, xbar_cols=8, flags=xo.WIRE_AAM2, r_row=0.0, r_col=0.0)
    assert np.allclose(xo.planes(aam0, W, 1.0), xo.planes(ideal, W, 1.0), rtol=0, atol=1e-12)


@pytest.mark.parametrize("R,C,rows,cols", [(5, 7, 5, 7), (8, 4, 8, 4), (6, 6, 4, 5)])
def test_aam2_first_order_coefficients_match_exact_circuit(xo, R, C, rows, cols):
    # With all wire resistances scaled by eps, d(plane)/d(eps) at 0 of the exact circuit holds the
    # weight of every shared segment (row prefix, column suffix, source, sense): a wrong index or a
    # dropped term anywhere changes it by O(1).  Partial tile: absent devices carry no current.
    rng = np.random.default_rng(R * 100 + C)
    d = rng.integers(0, 4, size=(rows, cols))
    base = dict(xbar_rows=R, xbar_cols=C, weight_bits=2, slice_bits=2, r_min=1e3, r_max=1e4)
    wires = dict(r_row=2.0, r_col=7.0, r_source=11.0, r_sense=13.0)
    eps = 1e-4
    cfg = xo.make_config(flags=xo.WIRE_AAM2, **base, **{k: v * eps for k, v in wires.items()})
    U = xo.planes(cfg, (d / 3.0).astype(np.float32), 1.0)[0]
    ref = xo.make_config(**base, **wires)
    slope_model = (U - d) / eps
    slope_exact = (_exact_plane(ref, d, rows, cols, scale=eps) - d) / eps
    assert np.abs(slope_exact).max() > 0.05
    assert np.abs(slope_model - slope_exact).max() < 2e-3 * np.abs(slope_exact).max()


@pytest.mark.parametrize("R,C", [(8, 8), (16, 16), (12, 5)])
def test_aam2_error_is_second_order_and_far_below_single_path_model(xo, R, C):
    rng = np.random.default_rng(R + C)
    d = rng.integers(0, 4, size=(R, C))
    W = (d / 3.0).astype(np.float32)
    errs2, errs1 = [], []
    for scale in (4.0, 2.0, 1.0):
        kw = dict(xbar_rows=R, xbar_cols=C, weight_bits=2, slice_bits=2, r_min=1e4, r_max=1e5,
                  r_row=1.0 * scale, r_col=4.6 * scale, r_source=3.0 * scale, r_sense=2.0 * scale)
        exact = _exact_plane(xo.make_config(**kw), d)
        errs2.append(np.abs(xo.planes(xo.make_config(flags=xo.WIRE_AAM2, **kw), W, 1.0)[0] - exact).max())
        errs1.append(np.abs(xo.planes(xo.make_config(flags=xo.WIRE_AAM, **kw), W, 1.0)[0] - exact).max())
    assert errs2[0] / errs2[1] > 3.0 and errs2[1] / errs2[2] > 3.0       # ~ eps^2
    assert 1.6 < errs1[1] / errs1[2] < 2.4                               # single path: first order remains
    assert errs2[2] < 0.05 * errs1[2]


def test_aam2_signed_weights_and_slices(xo):
    # sign symmetry and slice independence: each slice / polarity array is its own circuit
    R = C = 6
    rng = np.random.default_rng(9)
    q = rng.integers(-15, 16, size=(R, C))
    cfg = xo.make_config(xbar_rows=R, xbar_cols=C, weight_bits=4, slice_bits=2, flags=xo.WIRE_AAM2,
                         r_min=1e4, r_max=1e5, r_row=5.0, r_col=9.0)
    U = xo.planes(cfg, (q / 15.0).astype(np.float32), 1.0)
    assert np.array_equal(xo.planes(cfg, (-q / 15.0).astype(np.float32), 1.0), -U)
    dg = _device_g(cfg, 1) - _device_g(cfg, 0)
    for s in range(2):
        dig = (np.abs(q) >> (2 * s)) & 3
        Gp = _device_g(cfg, np.where(q > 0, dig, 0).astype(np.float64))
        Gn = _device_g(cfg, np.where(q < 0, dig, 0).astype(np.float64))
        exact = (nodal.effective_conductance(Gp, 5.0, 9.0) - nodal.effective_conductance(Gn, 5.0, 9.0)) / dg
        assert np.abs(U[s] - exact).max() < 2e-4


def test_nodal_solver_basics():
    # two cells on one column: hand-solved ladder.  Row drivers 1 V each, r_row a, r_col b.
    g1, g2, a, b = 1e-3, 2e-3, 5.0, 7.0
    E = nodal.effective_conductance([[g1], [g2]], a, b)
    # unknown column node voltages v1 (row 0), v2 (row 1): KCL by hand
    r1, r2 = 1 / g1 + a, 1 / g2 + a
    A = np.array([[1 / r1 + 1 / b, -1 / b], [-1 / b, 1 / r2 + 1 / b + 1 / b]])
    for drive in ((1.0, 0.0), (0.0, 1.0)):
        v = np.linalg.solve(A, np.array([drive[0] / r1, drive[1] / r2]))
        assert abs(v[1] / b - (E[0, 0] * drive[0] + E[1, 0] * drive[1])) < 1e-15
    rng = np.random.default_rng(0)
    G = rng.uniform(1e-6, 1e-5, size=(3, 4))
    # with wires of (almost) zero resistance the map is G itself
    assert np.allclose(nodal.effective_conductance(G, 1e-9, 1e-9), G, rtol=1e-6)


def test_sparse_nodal_solver_equals_dense_and_is_reciprocal():
    rng = np.random.default_rng(4)
    for R, C in ((1, 1), (2, 5), (12, 9), (16, 16)):
        G = rng.uniform(1e-6, 1e-4, size=(R, C))
        G[rng.random(size=(R, C)) < 0.2] = 0.0          # absent devices
        wires = (1.5, 4.6, 3.0, 2.0)
        dense = nodal.effective_conductance(G, *wires)
        sparse = nodal.effective_conductance_sparse(G, *wires)
        assert np.abs(dense - sparse).max() <= 1e-12 * np.abs(dense).max()
        # reciprocity of a passive network: drive the columns from the sense end and read the rows at
        # the driver end (wires and terminations swap roles, both index directions reverse)
        swapped = nodal.effective_conductance_sparse(G[::-1, ::-1].T, wires[1], wires[0], wires[3], wires[2])
        assert np.abs(swapped[::-1, ::-1].T - sparse).max() <= 1e-12 * np.abs(sparse).max()


def test_fcm_profile_closed_forms_and_layout(xo):
    from oracle import fcm
    # one device per tile: series connection
    kw = dict(weight_bits=4, slice_bits=2, r_row=30.0, r_col=500.0, r_source=1e3, r_sense=2e3, r_min=1e4, r_max=1e5)
    cfg = xo.make_config(xbar_rows=1, xbar_cols=1, **kw)
    q = np.array([[7, -9], [0, 15]])
    D = fcm.fcm_profile(cfg, (q / 15.0).astype(np.float32), 1.0)
    rho = 1e3 + 30.0 + 500.0 + 2e3
    for k in range(2):
        for n in range(2):
            for s in range(2):
                dig = (abs(int(q[k, n])) >> (2 * s)) & 3
                for pol in range(2):
                    on = (q[k, n] > 0) if pol == 0 else (q[k, n] < 0)
                    g = _device_g(cfg, dig if on else 0)
                    assert abs(D[s, pol, k, n] - (1.0 - 1.0 / (1.0 + rho * g))) < 1e-12
    # stored profile applied by the generator == exact circuit, tile by tile (ragged: 7 x 5 in 4 x 4 tiles)
    rng = np.random.default_rng(8)
    cfg = xo.make_config(xbar_rows=4, xbar_cols=4, flags=xo.WIRE_PROFILE, **kw)
    q = rng.integers(-15, 16, size=(7, 5))
    W = (q / 15.0).astype(np.float32)
    D = fcm.fcm_profile(cfg, W, 1.0)
    U = xo.planes(cfg, W, 1.0, profile=D.astype(np.float32))
    dg = _device_g(cfg, 1) - _device_g(cfg, 0)
    for s in range(2):
        dig = (np.abs(q) >> (2 * s)) & 3
        for k0 in range(0, 7, 4):
            for n0 in range(0, 5, 4):
                E = []
                for sign in (1, -1):
                    tile = np.zeros((4, 4))
                    blk = np.where(sign * q > 0, dig, 0)[k0:k0 + 4, n0:n0 + 4]
                    tile[:blk.shape[0], :blk.shape[1]] = _device_g(cfg, blk.astype(np.float64))
                    E.append(nodal.effective_conductance(tile, 30.0, 500.0, 1e3, 2e3)[:blk.shape[0], :blk.shape[1]])
                want = (E[0] - E[1]) / dg
                got = U[s, k0:k0 + 4, n0:n0 + 4]
                assert np.abs(got - want).max() < 1e-6     # profile passes through float32
    # no wire resistance to speak of: no distortion
    cfg0 = xo.make_config(xbar_rows=4, xbar_cols=4, weight_bits=4, slice_bits=2, r_row=1e-9, r_col=1e-9)
    assert np.abs(fcm.fcm_profile(cfg0, W, 1.0)).max() < 1e-10


def test_profile_mode_round_trip(xo):
    # D = (G_ideal - G_nonideal) / G_ideal taken from the analytical model reproduces its planes
    R, C, K, N, S = 8, 8, 20, 13, 4
    rng = np.random.default_rng(9)
    W = rng.uniform(-1, 1, size=(K, N)).astype(np.float32)
    aam = xo.make_config(xbar_rows=R, xbar_cols=C, flags=xo.WIRE_AAM, r_min=1e4, r_max=1e5)
    prof = xo.make_config(xbar_rows=R, xbar_cols=C, flags=xo.WIRE_PROFILE, r_min=1e4, r_max=1e5)
    D = np.zeros((S, 2, K, N), dtype=np.float32)
    for k in range(K):
        for n in range(N):
            rho = (n % C + 1) * 1.0 + (R - k % R) * 4.6
            qv = xo.quantize_weight(W[k, n], 1.0, 8)
            for s in range(S):
                d = (abs(qv) >> (2 * s)) & 3
                for pol in range(2):
                    g = _device_g(aam, d if (qv > 0) == (pol == 0) and qv != 0 else 0)
                    D[s, pol, k, n] = (g - g / (1 + rho * g)) / g
    Ua, Up = xo.planes(aam, W, 1.0), xo.planes(prof, W, 1.0, profile=D)
    assert np.allclose(Ua, Up, rtol=0, atol=3e-6)                    # D is stored in single precision
    zero = xo.planes(prof, W, 1.0, profile=np.zeros_like(D))
    assert np.allclose(zero, xo.planes(xo.make_config(xbar_rows=R, xbar_cols=C), W, 1.0), atol=1e-12)


def test_variation_statistics(xo):
    K, N = 64, 64
    W = np.full((K, N), 2.0 / 3.0, dtype=np.float32)                  # single slice, digit 2 everywhere
    cfg = xo.make_config(xbar_rows=64, xbar_cols=64, weight_bits=2, slice_bits=2, flags=xo.VARIATION,
                         var_sigma=0.1, seed=5)
    dg = (1e-5 - 1e-6) / 3
    U = xo.planes(cfg, W, 1.0, step=1)[0]
    res = (U - 2.0).ravel()
    sd = 0.1 * math.sqrt(_device_g(cfg, 2) ** 2 + _device_g(cfg, 0) ** 2) / dg
    assert abs(res.mean()) < 4 * sd / math.sqrt(res.size)
    assert abs(res.std() / sd - 1) < 0.05
    assert stats.kstest(res / sd, "norm").pvalue > 1e-3
    assert np.array_equal(U, xo.planes(cfg, W, 1.0, step=1)[0])       # same step: same draw
    assert not np.any(U == xo.planes(cfg, W, 1.0, step=2)[0])         # resampled per step
    # sub-block addressed by absolute indices sees the same devices
    k_idx, n_idx = np.array([3, 17, 40]), np.array([0, 5, 63, 21])
    Usub = xo.planes(cfg, W[np.ix_(k_idx, n_idx)], 1.0, step=1, k_idx=k_idx, n_idx=n_idx, K_full=K, N_full=N)[0]
    assert np.array_equal(Usub, U[np.ix_(k_idx, n_idx)])


def test_nonideal_bwd_is_fwd_through_transposed_tiles(xo):
    # reciprocity: the backward pass drives the same devices from the other side
    R, C, K, N, M = 8, 16, 21, 37, 5
    rng = np.random.default_rng(4)
    W = rng.normal(0, 0.3, size=(K, N)).astype(np.float32)
    dY = rng.normal(0, 0.01, size=(M, N)).astype(np.float32)
    kw = dict(weight_bits=8, slice_bits=2, input_bits=8, stream_bits=2, adc_bits=8, var_sigma=0.05,
              adc_fs_fwd=70.0, adc_fs_bwd=90.0, seed=3)
    cfg = xo.make_config(xbar_rows=R, xbar_cols=C, flags=xo.WIRE_AAM | xo.VARIATION, **kw)
    U = xo.planes(cfg, W, 1.0, step=2)
    dX, codes = xo.bwd_planes(cfg, U, dY, 1.0, 0.04, want_codes=True)
    kw["adc_fs_fwd"] = 90.0
    swapped = xo.make_config(xbar_rows=C, xbar_cols=R, flags=xo.INPUT_SIGNED, **kw)
    Y2, codes2 = xo.fwd_planes(swapped, np.ascontiguousarray(U.transpose(0, 2, 1)), dY, 1.0, 0.04, want_codes=True)
    assert np.array_equal(dX, Y2) and np.array_equal(codes, codes2)
    # and it is close to the exact product when the ADC is fine enough
    fine = xo.make_config(xbar_rows=R, xbar_cols=C, flags=0, **dict(kw, adc_bits=12, adc_fs_bwd=16 * 3 * 3.0))
    dXf = xo.bwd(fine, W, dY, 1.0, 0.04)
    ref = dY.astype(np.float64) @ W.astype(np.float64).T
    assert np.linalg.norm(dXf - ref) < 0.05 * np.linalg.norm(ref)


def test_tiny_fwd_brute_force(xo):
    """Everything at once on a 2-tile problem, re-derived device by device with exact fractions of
    the physical quantities (series path per device, two arrays, subtract, threshold search)."""
    R, C, K, N, M = 4, 4, 6, 5, 3
    cfg = xo.make_config(xbar_rows=R, xbar_cols=C, weight_bits=4, slice_bits=2, input_bits=4, stream_bits=2,
                         adc_bits=5, flags=xo.WIRE_AAM | xo.INPUT_SIGNED, r_min=2e3, r_max=2e4, r_row=3.0,
                         r_col=9.0, adc_fs_fwd=20.0, adc_fs_bwd=20.0)
    rng = np.random.default_rng(12)
    qv = rng.integers(-15, 16, size=(K, N))
    av = rng.integers(-15, 16, size=(M, K))
    W, X = (qv / 15.0).astype(np.float32), (av / 15.0).astype(np.float32)
    Y, codes, acc = xo.fwd(cfg, W, X, 1.0, 1.0, want_codes=True, want_acc=True)
    g_lo, g_hi = 1 / 2e4, 1 / 2e3
    dg = (g_hi - g_lo) / 3
    gain = float(np.float32(15.0) / np.float32(20.0))
    total = np.zeros((M, N))
    for m in range(M):
        for n in range(N):
            for p, sgn in ((0, 1), (1, -1)):
                for b in range(2):
                    for s in range(2):
                        for t in range(2):
                            cur = 0.0
                            for k in range(t * R, min(K, t * R + R)):
                                a = av[m, k] * sgn
                                dig_in = ((a if a > 0 else 0) >> (2 * b)) & 3
                                dig_w = (abs(int(qv[k, n])) >> (2 * s)) & 3
                                rho = (n % C + 1) * 3.0 + (R - k % R) * 9.0
                                r_act = 1.0 / (g_lo + dig_w * dg) + rho
                                r_rest = 1.0 / g_lo + rho
                                i_pos = dig_in / (r_act if qv[k, n] > 0 else r_rest)
                                i_neg = dig_in / (r_act if qv[k, n] < 0 else r_rest)
                                cur += (i_pos - i_neg) / dg
                            x = cur * gain
                            code = min(range(-15, 16), key=lambda c: (abs(x - c), c % 2))   # nearest, even on ties
                            assert codes[p, b, s, t, m, n] == code
                            total[m, n] += sgn * (1 << (2 * s + 2 * b)) * code
    assert np.array_equal(acc, total.astype(np.int64))
    assert np.allclose(Y, total * (20.0 / 15) / (15 * 15), rtol=1e-6, atol=0)


def test_dac_table(xo):
    # a linear table equals the ideal DAC; a scaled table scales the currents
    rng = np.random.default_rng(6)
    W = rng.uniform(-1, 1, size=(16, 8)).astype(np.float32)
    X = rng.uniform(0, 1, size=(4, 16)).astype(np.float32)
    kw = dict(xbar_rows=8, xbar_cols=8, input_bits=8, stream_bits=2, adc_bits=12, adc_fs_fwd=8 * 9.0)
    base = xo.fwd(xo.make_config(**kw), W, X, 1.0, 1.0)
    lin = xo.fwd(xo.make_config(flags=xo.DAC_LUT, dac_lut=[0, 1 / 3, 2 / 3, 1.0], **kw), W, X, 1.0, 1.0)
    assert np.array_equal(base, lin)
    half = xo.fwd(xo.make_config(flags=xo.DAC_LUT, dac_lut=[0, 1 / 6, 2 / 6, 0.5], **dict(kw, adc_fs_fwd=4 * 9.0)),
                  W, X, 1.0, 1.0, want_codes=True)[1]
    full = xo.fwd(xo.make_config(**kw), W, X, 1.0, 1.0, want_codes=True)[1]
    assert np.abs(half - full).max() <= 1


def test_adc_range_rule_rarely_saturates(xo):
    # the stand-in ADC range of the workload recipe clips only a small fraction of conversions
    g = workloads.Gemm("t", 256, 48, 8, False, 1)
    W, X, _ = workloads.layer_tensors_np(g, 3)
    kw = workloads.config_kwargs("resnet50")
    kw["flags"] = kw["flags"] & ~(workloads.NI_UPD_NL | workloads.NI_UPD_NOISE)
    cfg = xo.make_config(**kw)
    codes = xo.fwd(cfg, W, X, float(np.abs(W).max()), float(X.max()), want_codes=True)[1]
    assert (np.abs(codes) == 127).mean() < 0.01


# ------------------------------------------------------------------------------------------------
# update model
# ------------------------------------------------------------------------------------------------
def _upd_tensors(seed, M=7, K=9, N=5):
    rng = np.random.default_rng(seed)
    W = rng.uniform(-0.4, 0.4, size=(K, N)).astype(np.float32)
    X = rng.uniform(0, 1, size=(M, K)).astype(np.float32)
    dY = rng.normal(0, 0.01, size=(M, N)).astype(np.float32)
    return W, X, dY


def test_update_ideal_is_plain_sgd(xo):
    W, X, dY = _upd_tensors(0)
    cfg = xo.make_config(flags=0)
    W2, grad = xo.update(cfg, W, X, dY, w_max=0.5, grad_scale=2.0, lr=0.1, want_grad=True)
    ref_grad = X.astype(np.float64).T @ dY.astype(np.float64)
    assert np.allclose(grad, ref_grad, rtol=1e-13, atol=1e-18)
    ref = W.astype(np.float64) - 0.5 * 0.1 * 2.0 * ref_grad        # dW = -lr * w_max * grad_scale * grad
    assert np.allclose(W2, ref, rtol=0, atol=1e-7)
    # the switched-off factors must not matter
    cfg0 = xo.make_config(flags=xo.UPD_NL | xo.UPD_NOISE, upd_nl_v=0.0, upd_noise_gamma=0.0)
    assert np.array_equal(W2, xo.update(cfg0, W, X, dY, 0.5, 2.0, 0.1))


def test_update_clamps_to_device_range(xo):
    W, X, dY = _upd_tensors(1)
    W2 = xo.update(xo.make_config(flags=0), W, X, dY * 1e4, w_max=0.5, grad_scale=50.0, lr=1.0)
    assert np.abs(W2).max() <= 0.5 and (np.abs(W2) == 0.5).any()


def test_update_nonlinearity_closed_forms(xo):
    v = 0.7
    cfg = xo.make_config(flags=xo.UPD_NL, upd_nl_v=v)
    X = np.ones((1, 1), dtype=np.float32)
    lr, gs, w_max = 0.25, 1.0, 1.0
    for g0, x in ((-1.0, 0.0), (1.0, 1.0), (0.0, 0.5), (0.5, 0.75)):
        for grad in (0.2, -0.2):
            W = np.array([[g0]], dtype=np.float32)
            dY = np.array([[grad]], dtype=np.float32)
            W2 = xo.update(cfg, W, X, dY, w_max, gs, lr)
            delta = float(np.float32(grad))
            up = -lr * delta > 0
            factor = math.exp(-v * x) if up else math.exp(-v * (1 - x))
            expect = min(1.0, max(-1.0, g0 - lr * delta * factor))
            assert abs(float(W2[0, 0]) - expect) < 1e-7
    # mirror symmetry: state g with gradient d moves like state -g with gradient -d, mirrored
    for g0 in (-0.6, 0.1, 0.8):
        a = xo.update(cfg, np.array([[g0]], np.float32), X, np.array([[0.3]], np.float32), 1.0, 1.0, 0.2)
        b = xo.update(cfg, np.array([[-g0]], np.float32), X, np.array([[-0.3]], np.float32), 1.0, 1.0, 0.2)
        assert abs(float(a[0, 0]) + float(b[0, 0])) < 1e-7
    # small v barely matters, large v does (the paper's sensitivity trend)
    W, Xr, dY = _upd_tensors(2)
    sgd = xo.update(xo.make_config(flags=0), W, Xr, dY, 0.5, 1.0, 0.5)
    small = xo.update(xo.make_config(flags=xo.UPD_NL, upd_nl_v=0.01), W, Xr, dY, 0.5, 1.0, 0.5)
    large = xo.update(xo.make_config(flags=xo.UPD_NL, upd_nl_v=1.0), W, Xr, dY, 0.5, 1.0, 0.5)
    step = np.abs(sgd - W).max()
    assert np.abs(small - sgd).max() < 0.011 * step < np.abs(large - sgd).max()


def test_update_noise_statistics(xo):
    K, N, M = 100, 80, 1
    gamma, lr, gs = 5.0, 0.01, 1.0
    cfg = xo.make_config(flags=xo.UPD_NOISE, upd_noise_gamma=gamma, seed=9)
    W = np.zeros((K, N), dtype=np.float32)
    X = np.ones((M, K), dtype=np.float32)
    for grad in (1e-4, 4e-4):
        dY = np.full((M, N), grad, dtype=np.float32)
        W2 = xo.update(cfg, W, X, dY, 1.0, gs, lr, step=4)
        delta = float(np.float32(grad))
        dev = (W2.astype(np.float64) - (0.0 - lr * delta)).ravel()
        sd = lr * gamma * math.sqrt(delta)                           # sigma grows like sqrt(|delta|)
        assert abs(dev.mean()) < 4 * sd / 100
        assert abs(dev.std() / sd - 1) < 0.03
        assert stats.kstest(dev / sd, "norm").pvalue > 1e-3
    # weight (k, n) of a layer with N columns consumes normal number k * N + n of the write stream
    z = xo.normals(9, xo.STREAM_WRITE, 4, 0, K * N).reshape(K, N)
    assert np.allclose(-dev.reshape(K, N) / sd, z, rtol=0, atol=2e-4)   # W = g - lr * (delta + sigma z)
    assert np.array_equal(W2, xo.update(cfg, W, X, dY, 1.0, gs, lr, step=4))
    assert not np.any(W2 == xo.update(cfg, W, X, dY, 1.0, gs, lr, step=5))
    # a sub-block addressed by absolute indices draws the same numbers
    k_idx, n_idx = np.array([5, 50, 99]), np.array([0, 7, 78, 33])
    sub = xo.update(cfg, W[np.ix_(k_idx, n_idx)], X[:, k_idx], dY[:, n_idx], 1.0, gs, lr, step=4,
                    k_idx=k_idx, n_idx=n_idx, N_full=N)
    assert np.array_equal(sub, W2[np.ix_(k_idx, n_idx)])


# ------------------------------------------------------------------------------------------------
# convolution layers: patch gathering and its adjoint
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("B,H,W,C,k,stride,pad,N", [(2, 7, 6, 3, 3, 1, 1, 5), (1, 9, 9, 4, 3, 2, 1, 2),
                                                    (2, 8, 8, 5, 1, 2, 0, 3), (1, 11, 10, 3, 7, 2, 3, 4)])
def test_im2col_matmul_is_the_library_convolution(B, H, W, C, k, stride, pad, N):
    import torch
    from oracle import conv
    rng = np.random.default_rng(B * 100 + H)
    X = rng.normal(size=(B, H, W, C))
    Wm = rng.normal(size=(k * k * C, N))                    # rows ordered (kh, kw, c)
    Y = conv.im2col(X, k, k, stride, pad) @ Wm
    OH, OW = conv.out_size(H, k, stride, pad), conv.out_size(W, k, stride, pad)
    w_torch = torch.from_numpy(Wm.reshape(k, k, C, N)).permute(3, 2, 0, 1)         # [N][C][kh][kw]
    ref = torch.nn.functional.conv2d(torch.from_numpy(X).permute(0, 3, 1, 2), w_torch, stride=stride, padding=pad)
    assert np.allclose(Y.reshape(B, OH, OW, N), ref.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)
    # col2im is the adjoint: <im2col(x), y> == <x, col2im(y)>, and equals the library's fold
    Z = rng.normal(size=(B * OH * OW, k * k * C))
    back = conv.col2im(Z, X.shape, k, k, stride, pad)
    assert abs(np.vdot(conv.im2col(X, k, k, stride, pad), Z) - np.vdot(X, back)) < 1e-9
    zt = torch.from_numpy(Z.reshape(B, OH * OW, k, k, C)).permute(0, 4, 2, 3, 1).reshape(B, C * k * k, OH * OW)
    fold = torch.nn.functional.fold(zt, (H, W), kernel_size=k, stride=stride, padding=pad)
    assert np.allclose(back, fold.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)


# ------------------------------------------------------------------------------------------------
# digital peripherals: definitions against the library's functions and its automatic differentiation
# ------------------------------------------------------------------------------------------------
def test_peripheral_definitions_against_library_autograd():
    import torch
    from oracle import periph
    rng = np.random.default_rng(11)
    B, H, W, C = 3, 6, 5, 7
    x = rng.normal(size=(B, H, W, C))
    dy = rng.normal(size=(B, H, W, C))
    gamma, beta = rng.uniform(0.5, 1.5, size=C), rng.normal(size=C)
    # batch normalisation (training mode)
    xt = torch.tensor(x, requires_grad=True)
    gt, bt = torch.tensor(gamma, requires_grad=True), torch.tensor(beta, requires_grad=True)
    yt = torch.nn.functional.batch_norm(xt.permute(0, 3, 1, 2), None, None, gt, bt, training=True, eps=1e-5)
    yt.backward(torch.tensor(dy).permute(0, 3, 1, 2))
    y, mean, invstd = periph.bn_fwd(x, gamma, beta, 1e-5)
    dx, dgamma, dbeta = periph.bn_bwd(x, dy, gamma, mean, invstd)
    assert np.allclose(y, yt.detach().permute(0, 2, 3, 1).numpy(), atol=1e-12)
    assert np.allclose(dx, xt.grad.numpy(), atol=1e-12)
    assert np.allclose(dgamma, gt.grad.numpy(), atol=1e-12) and np.allclose(dbeta, bt.grad.numpy(), atol=1e-12)
    # ReLU
    xt = torch.tensor(x, requires_grad=True)
    rt = torch.relu(xt)
    rt.backward(torch.tensor(dy))
    assert np.array_equal(periph.relu_fwd(x), rt.detach().numpy())
    assert np.array_equal(periph.relu_bwd(periph.relu_fwd(x), dy), xt.grad.numpy())
    # sigmoid against autograd, and its closed-form properties
    xt = torch.tensor(x, requires_grad=True)
    st = torch.sigmoid(xt)
    st.backward(torch.tensor(dy))
    assert np.allclose(periph.sigmoid_fwd(x), st.detach().numpy(), atol=1e-15)
    assert np.allclose(periph.sigmoid_bwd(periph.sigmoid_fwd(x), dy), xt.grad.numpy(), atol=1e-15)
    assert periph.sigmoid_fwd(0.0) == 0.5 and np.allclose(periph.sigmoid_fwd(x) + periph.sigmoid_fwd(-x), 1.0, atol=1e-15)
    # max pooling 3x3 stride 2 pad 1 and 2x2 stride 2
    for k, stride, pad in ((3, 2, 1), (2, 2, 0)):
        xt = torch.tensor(x, requires_grad=True)
        pt = torch.nn.functional.max_pool2d(xt.permute(0, 3, 1, 2), k, stride, pad)
        d = rng.normal(size=tuple(pt.permute(0, 2, 3, 1).shape))
        pt.backward(torch.tensor(d).permute(0, 3, 1, 2))
        y, arg = periph.maxpool_fwd(x, k, stride, pad)
        assert np.array_equal(y, pt.detach().permute(0, 2, 3, 1).numpy())
        assert np.allclose(periph.maxpool_bwd(d, arg, x.shape), xt.grad.numpy(), atol=1e-12)
    # global average pooling
    xt = torch.tensor(x, requires_grad=True)
    at = xt.mean(dim=(1, 2))
    d = rng.normal(size=(B, C))
    at.backward(torch.tensor(d))
    assert np.allclose(periph.avgpool_fwd(x), at.detach().numpy(), atol=1e-12)
    assert np.allclose(periph.avgpool_bwd(d, x.shape), xt.grad.numpy(), atol=1e-12)
    # softmax cross-entropy, mean over the batch
    z = rng.normal(size=(5, 10)) * 3
    labels = rng.integers(0, 10, size=5)
    zt = torch.tensor(z, requires_grad=True)
    lt = torch.nn.functional.cross_entropy(zt, torch.tensor(labels), reduction="none")
    lt.mean().backward()
    loss, dz = periph.softmax_xent(z, labels, 1.0 / 5)
    assert np.allclose(loss, lt.detach().numpy(), atol=1e-12) and np.allclose(dz, zt.grad.numpy(), atol=1e-12)


# ------------------------------------------------------------------------------------------------
# pulse-level update (stochastic pulse trains)
# ------------------------------------------------------------------------------------------------
def _train_from_philox(xo, seed, stream, step, index, p, bl):
    """The documented construction, from the Philox function alone."""
    key = [(seed & 0xFFFFFFFF) ^ ((0x9E3779B9 * stream) & 0xFFFFFFFF), (seed >> 32) ^ ((0xBB67AE85 * stream) & 0xFFFFFFFF)]
    thr = int(np.rint(min(max(p, 0.0), 1.0) * 4294967296.0))
    bits = 0
    for j in range(bl):
        blk = index * 8 + j // 4
        w = xo.philox4x32_10([blk & 0xFFFFFFFF, blk >> 32, step & 0xFFFFFFFF, step >> 32], key)
        if w[j % 4] < thr:
            bits |= 1 << j
    return bits


def test_pulse_trains(xo):
    seed = 0x1234567890ABCDEF
    for bl in (1, 10, 31):
        full = (1 << bl) - 1
        assert xo.pulse_train(seed, 3, 7, 11, 0.0, bl) == 0
        assert xo.pulse_train(seed, 3, 7, 11, 1.0, bl) == full and xo.pulse_train(seed, 3, 7, 11, 2.5, bl) == full
        for index, p in ((0, 0.5), (123456789012, 0.3), (5, 0.999)):
            t = xo.pulse_train(seed, 4, 9, index, p, bl)
            assert t == _train_from_philox(xo, seed, 4, 9, index, p, bl) and t <= full
    # a longer train extends a shorter one; rows and columns, steps and elements draw different trains
    assert xo.pulse_train(seed, 3, 0, 5, 0.5, 31) & 0x3FF == xo.pulse_train(seed, 3, 0, 5, 0.5, 10)
    base = xo.pulse_train(seed, 3, 0, 5, 0.5, 31)
    assert len({base, xo.pulse_train(seed, 4, 0, 5, 0.5, 31), xo.pulse_train(seed, 3, 1, 5, 0.5, 31),
                xo.pulse_train(seed, 3, 0, 6, 0.5, 31)}) == 4
    # firing frequency = p (4 sigma over 31 * 3000 slots)
    for p in (0.1, 0.5, 0.83):
        ones = sum(bin(xo.pulse_train(seed, 3, 2, i, p, 31)).count("1") for i in range(3000))
        n = 31 * 3000
        assert abs(ones - n * p) <= 4 * np.sqrt(n * p * (1 - p))


def test_pulsed_update_counts_and_linear_device(xo):
    rng = np.random.default_rng(8)
    M, K, N, bl, dw = 9, 7, 5, 31, 2.0 ** -12
    X = rng.uniform(-1.2, 1.2, size=(M, K)).astype(np.float32)
    dY = rng.uniform(-0.5, 0.5, size=(M, N)).astype(np.float32)
    W0 = rng.uniform(-0.5, 0.5, size=(K, N)).astype(np.float32)
    cfg = xo.make_config(seed=77)
    W1, pulses = xo.update_pulsed(cfg, W0, X, dY, 2.0, 1.0, 0.4, bl, dw, step=3, want_pulses=True)
    # brute force: trains from the Philox function, coincidences, direction against the sign of x d
    want = np.zeros((K, N), dtype=np.int64)
    for m in range(M):
        a = [_train_from_philox(xo, 77, 3, 3, m * K + k, abs(float(X[m, k])) / 1.0, bl) for k in range(K)]
        b = [_train_from_philox(xo, 77, 4, 3, m * N + n, abs(float(dY[m, n])) / np.float64(np.float32(0.4)), bl) for n in range(N)]
        for k in range(K):
            for n in range(N):
                c = bin(a[k] & b[n]).count("1")
                want[k, n] -= c * int(np.sign(X[m, k]) * np.sign(dY[m, n]))
    assert np.array_equal(pulses, want) and np.abs(want).max() > 3
    # linear device: every pulse moves the state by dw_min (all quantities here are exact in binary)
    assert np.array_equal(W1, (W0.astype(np.float64) + 2.0 * dw * want).astype(np.float32))
    # values at the range: every slot fires on both sides, bl pulses per sample
    Xf, Df = np.full((4, 2), 1.0, np.float32), np.array([[0.4, -0.4, 1.0]] * 4, dtype=np.float32)
    _, p = xo.update_pulsed(cfg, np.zeros((2, 3), np.float32), Xf, Df, 2.0, 1.0, 0.4, bl, dw, want_pulses=True)
    assert np.array_equal(p, np.array([[-4 * bl, 4 * bl, -4 * bl]] * 2))
    # zero inputs or zero errors: nothing is written
    assert np.array_equal(xo.update_pulsed(cfg, W0, 0 * X, dY, 2.0, 1.0, 0.4, bl, dw), W0)
    assert np.array_equal(xo.update_pulsed(cfg, W0, X, 0 * dY, 2.0, 1.0, 0.4, bl, dw), W0)


def test_pulsed_update_is_unbiased_outer_product(xo):
    """Expected pulses = bl p_x p_d: the mean written change is the outer-product update."""
    rng = np.random.default_rng(9)
    M, K, N, bl = 6000, 4, 3, 31
    X = rng.uniform(-1, 1, size=(M, K)).astype(np.float32)
    dY = rng.uniform(-1, 1, size=(M, N)).astype(np.float32)
    _, pulses = xo.update_pulsed(xo.make_config(seed=5), np.zeros((K, N), np.float32), X, dY, 1.0, 1.0, 1.0, bl, 1e-6,
                                 want_pulses=True)
    px, pd = np.abs(X.astype(np.float64)), np.abs(dY.astype(np.float64))
    mean = -bl * (X.astype(np.float64).T @ dY.astype(np.float64))
    # variance of a coincidence count: bl p (1 - p) with p = px pd, independent over samples
    pp = px[:, :, None] * pd[:, None, :]
    sigma = np.sqrt((bl * pp * (1 - pp)).sum(axis=0))
    assert (np.abs(pulses - mean) <= 4.5 * sigma).all()
    assert np.abs(mean).max() > 20 * sigma.max() / 4.5            # the test can see a wrong factor or sign


def test_pulsed_update_of_sampled_devices(xo):
    """Devices are independent: updating the devices at some rows and columns of a layer gives exactly their
    entries of the whole layer's update (same trains, same noise numbers)."""
    rng = np.random.default_rng(31)
    M, K, N, bl, dw = 40, 23, 17, 31, 2.0 ** -9
    X = rng.uniform(-1.5, 1.5, size=(M, K)).astype(np.float32)
    dY = rng.uniform(-0.3, 0.3, size=(M, N)).astype(np.float32)
    W0 = rng.uniform(-0.5, 0.5, size=(K, N)).astype(np.float32)
    for flags in (0, xo.UPD_NL | xo.UPD_NOISE, xo.PULSE_CODED | xo.UPD_NOISE):
        cfg = xo.make_config(flags=flags, upd_nl_v=0.8, upd_noise_gamma=0.7, seed=13)
        W1, p1 = xo.update_pulsed(cfg, W0, X, dY, 1.2, 1.0, 0.2, bl, dw, step=4, want_pulses=True)
        ks, ns = np.array([0, 5, 22, 11]), np.array([16, 3, 4])
        Ws, ps = xo.update_pulsed(cfg, W0[np.ix_(ks, ns)], X[:, ks], dY[:, ns], 1.2, 1.0, 0.2, bl, dw, step=4, want_pulses=True,
                                  k_idx=ks, n_idx=ns, K_full=K, N_full=N)
        assert np.array_equal(ps, p1[np.ix_(ks, ns)]) and np.array_equal(Ws, W1[np.ix_(ks, ns)])
        assert np.abs(p1).max() > 5
        if not flags & xo.PULSE_CODED:      # without the positions the trains are other trains
            Wn, pn = xo.update_pulsed(cfg, W0[np.ix_(ks, ns)], X[:, ks], dY[:, ns], 1.2, 1.0, 0.2, bl, dw, step=4, want_pulses=True)
            assert not np.array_equal(pn, ps)


def test_coded_pulses_multiply(xo):
    """Deterministic pulse coding: rows hold whole frames, columns fire sub-slots of every frame, so a device
    sees (coded |x|) x (coded |d|) coincidences; on the coding grid the written change IS the outer product."""
    for bl, frames in ((31, (5, 6)), (30, (5, 6)), (16, (4, 4)), (15, (3, 5)), (1, (1, 1)), (3, (1, 3)), (4, (2, 2))):
        tx, td = xo.pulse_frames(bl)
        assert (tx, td) == frames and tx * td <= bl < (tx + 1) * (tx + 1)
        for px in np.linspace(0, 1.3, 14):
            for pd in np.linspace(0, 1.3, 11):
                a, b = xo.pulse_code(px, bl, False), xo.pulse_code(pd, bl, True)
                nx = int(np.rint(min(px, 1.0) * tx))            # rint: ties to even, like the coder
                nd = int(np.rint(min(pd, 1.0) * td))
                assert bin(a).count("1") == nx * td and bin(b).count("1") == nd * tx
                assert bin(a & b).count("1") == nx * nd and (a | b) < (1 << (tx * td))
    # on the grid, linear noise-free devices: the update equals the aggregate outer-product update at the
    # learning rate Tx Td dw_min w_max / (x_range d_range), with no randomness left
    rng = np.random.default_rng(12)
    M, K, N, bl, dw = 7, 5, 4, 31, 2.0 ** -12
    tx, td = 5, 6
    X = (rng.integers(-tx, tx + 1, size=(M, K)) / tx * 2.0).astype(np.float32)          # x_range 2
    D = (rng.integers(-td, td + 1, size=(M, N)) / td * 0.5).astype(np.float32)          # d_range 0.5
    W0 = rng.uniform(-0.3, 0.3, size=(K, N)).astype(np.float32)
    cfg = xo.make_config(flags=xo.PULSE_CODED, seed=3)
    W1, pulses = xo.update_pulsed(cfg, W0, X, D, 1.5, 2.0, 0.5, bl, dw, step=1, want_pulses=True)
    nx = np.rint(X.astype(np.float64) / 2.0 * tx).astype(np.int64)
    nd = np.rint(D.astype(np.float64) / 0.5 * td).astype(np.int64)
    assert np.array_equal(pulses, -(nx.T @ nd)) and np.abs(pulses).max() > 20
    assert np.array_equal(W1, (W0.astype(np.float64) + 1.5 * dw * pulses).astype(np.float32))
    lr = tx * td * dw * 1.5 / (2.0 * 0.5)
    Wa = xo.update(xo.make_config(), W0, X, D, 1.5, 1.0 / 1.5, lr)
    assert np.abs(W1.astype(np.float64) - Wa).max() < 1e-6
    # the seed and the step do not enter; values below half a level write nothing
    assert np.array_equal(xo.update_pulsed(xo.make_config(flags=xo.PULSE_CODED, seed=99), W0, X, D, 1.5, 2.0, 0.5, bl, dw, step=8), W1)
    tiny = xo.update_pulsed(cfg, W0, X * 0.09, D, 1.5, 2.0, 0.5, bl, dw)
    assert np.array_equal(tiny, W0)
    # per-pulse noise uses Tx Td slots in its learning rate (31 slots give 30 usable ones)
    cn = xo.make_config(flags=xo.PULSE_CODED | xo.UPD_NOISE, upd_noise_gamma=0.6, seed=21)
    Wn = xo.update_pulsed(cn, np.zeros((1, 1), np.float32), np.array([[2.0]], np.float32), np.array([[-0.5]], np.float32),
                          4.0, 2.0, 0.5, 31, dw, step=6)
    lr_eq, g = 30 * dw * 4.0 / (2.0 * 0.5), 0.0
    for j in range(30):
        g += dw + np.float64(np.float32(0.6)) * np.sqrt(lr_eq * dw) * xo.normal(21, 5, 6 << 31, j)
    assert abs(Wn[0, 0] - 4.0 * g) < 1e-6


def test_pulsed_update_device_model(xo):
    """Per-pulse non-linearity and noise: sequential closed forms, and the aggregate model for one pulse."""
    bl, dw, v, gamma = 31, 2.0 ** -9, 1.7, 0.6
    X, D = np.array([[1.0]], np.float32), np.array([[-1.0]], np.float32)         # x d < 0: bl pulses upwards
    for g0 in (-0.8, 0.1, 0.97):
        W0 = np.array([[g0]], np.float32)
        cfg = xo.make_config(flags=xo.UPD_NL, upd_nl_v=v)
        up = xo.update_pulsed(cfg, W0, X, D, 1.0, 1.0, 1.0, bl, dw)[0, 0]
        down = xo.update_pulsed(cfg, W0, X, -D, 1.0, 1.0, 1.0, bl, dw)[0, 0]
        gu = gd = float(W0[0, 0])
        for _ in range(bl):
            gu = min(gu + dw * np.exp(-np.float64(np.float32(v)) * (gu + 1) / 2), 1.0)
            gd = max(gd - dw * np.exp(-np.float64(np.float32(v)) * (1 - (gd + 1) / 2)), -1.0)
        assert abs(up - gu) < 1e-6 and abs(down - gd) < 1e-6
        assert up - g0 > 0 > down - g0
        # one pulse = the aggregate model writing the same ideal change (learning rate 1, delta = -+dw)
        one_up = xo.update_pulsed(cfg, W0, X, D, 1.0, 1.0, 1.0, 1, dw)[0, 0]
        agg_up = xo.update(cfg, W0, X, D, 1.0, dw, 1.0)[0, 0]
        assert abs(one_up - agg_up) < 1e-7
        one_dn = xo.update_pulsed(cfg, W0, X, -D, 1.0, 1.0, 1.0, 1, dw)[0, 0]
        agg_dn = xo.update(cfg, W0, X, -D, 1.0, dw, 1.0)[0, 0]
        assert abs(one_dn - agg_dn) < 1e-7
    # noise: pulse j of sample m of device dev takes normal number m*32 + j of stream 5 keyed (step << 31) | dev;
    # its size is gamma sqrt(lr dw_min) with lr = bl dw_min w_max / (x_range d_range), the learning rate at which
    # the aggregate update equals the mean of this scheme
    cfg = xo.make_config(flags=xo.UPD_NOISE, upd_noise_gamma=gamma, seed=21)
    K, N, step = 2, 3, 6
    Xn, Dn = np.full((2, K), 2.0, np.float32), np.full((2, N), -0.5, np.float32)       # at the ranges: every slot fires
    Wn = xo.update_pulsed(cfg, np.zeros((K, N), np.float32), Xn, Dn, 4.0, 2.0, 0.5, 3, dw, step=step)
    lr_eq = 3 * dw * 4.0 / (2.0 * 0.5)
    for k in range(K):
        for n in range(N):
            g = 0.0
            for m in range(2):
                for j in range(3):
                    g += dw + np.float64(np.float32(gamma)) * np.sqrt(lr_eq * dw) * xo.normal(21, 5, (step << 31) | (k * N + n), m * 32 + j)
                    g = min(max(g, -1.0), 1.0)
            assert abs(Wn[k, n] - 4.0 * g) < 1e-6
    # n pulses carry the noise the aggregate model gives their sum at that learning rate: the same change
    # written pulse by pulse and in one aggregate write has the same mean and the same spread over many devices
    K = N = 60
    bl, g5, xr, dr, wm = 16, 5.0, 1.0, 0.25, 1.0
    lr_eq = bl * dw * wm / (xr * dr)
    cn = xo.make_config(flags=xo.UPD_NOISE, upd_noise_gamma=g5, seed=2)
    ones, minus = np.ones((1, K), np.float32), -np.full((1, N), dr, np.float32)              # every slot fires: bl pulses up
    Wp = xo.update_pulsed(cn, np.zeros((K, N), np.float32), ones * xr, minus, wm, xr, dr, bl, dw).astype(np.float64)
    Wa = xo.update(cn, np.zeros((K, N), np.float32), ones * xr, minus, wm, 1.0 / wm, lr_eq).astype(np.float64)
    assert abs(Wp.mean() - bl * dw) < 5 * Wp.std() / K and abs(Wa.mean() - bl * dw) < 5 * Wa.std() / K
    assert abs(Wp.std() / Wa.std() - 1) < 0.06
    assert abs(Wa.std() / (g5 * np.sqrt(lr_eq * bl * dw)) - 1) < 0.06


def test_magnitude_coded_pulses(xo):
    """One pulse per sample whose height codes the value: the device writes lx ld quanta in ONE write."""
    rng = np.random.default_rng(31)
    M, K, N, bl, dw = 6, 5, 4, 7, 2.0 ** -14
    X = (rng.integers(-bl, bl + 1, size=(M, K)) / bl * 2.0).astype(np.float32)          # on the level grid, x_range 2
    D = (rng.integers(-bl, bl + 1, size=(M, N)) / bl * 0.5).astype(np.float32)          # d_range 0.5
    W0 = rng.uniform(-0.3, 0.3, size=(K, N)).astype(np.float32)
    cfg = xo.make_config(flags=xo.PULSE_MAGNITUDE, seed=3)
    W1, quanta = xo.update_pulsed(cfg, W0, X, D, 1.5, 2.0, 0.5, bl, dw, step=1, want_pulses=True)
    lx = np.rint(X.astype(np.float64) / 2.0 * bl).astype(np.int64)
    ld = np.rint(D.astype(np.float64) / 0.5 * bl).astype(np.int64)
    # quanta = product of the two heights, against the sign of x d, summed over the samples
    assert np.array_equal(quanta, -(lx.T @ ld)) and np.abs(quanta).max() > 20
    # linear noise-free device: the quanta are all that is written, and that is the aggregate outer-product
    # update at the learning rate bl^2 dw_min w_max / (x_range d_range)
    assert np.array_equal(W1, (W0.astype(np.float64) + 1.5 * dw * quanta).astype(np.float32))
    lr = bl * bl * dw * 1.5 / (2.0 * 0.5)
    assert np.abs(W1.astype(np.float64) - xo.update(xo.make_config(), W0, X, D, 1.5, 1.0 / 1.5, lr)).max() < 1e-6
    # the same heights as frames x sub-slots of the time-coded scheme (5 x 5 of 25 slots) give the same counts
    Xc = (rng.integers(-5, 6, size=(M, K)) / 5 * 2.0).astype(np.float32)
    Dc = (rng.integers(-5, 6, size=(M, N)) / 5 * 0.5).astype(np.float32)
    _, q_mag = xo.update_pulsed(cfg, W0, Xc, Dc, 1.5, 2.0, 0.5, 5, dw, want_pulses=True)
    _, q_time = xo.update_pulsed(xo.make_config(flags=xo.PULSE_CODED), W0, Xc, Dc, 1.5, 2.0, 0.5, 25, dw, want_pulses=True)
    assert np.array_equal(q_mag, q_time)
    # off the grid the heights round to the nearest level (ties to even), beyond the range they saturate;
    # seed and step do not enter a noise-free write
    x, d = np.array([[0.93], [5.0], [0.1]], np.float32), np.array([[0.31], [-0.2], [0.01]], np.float32)
    _, q = xo.update_pulsed(xo.make_config(flags=xo.PULSE_MAGNITUDE, seed=77), np.zeros((1, 1), np.float32), x, d, 1.0, 2.0, 0.5,
                            bl, dw, step=9, want_pulses=True)
    want = -(int(np.rint(0.93 / 2 * 7)) * int(np.rint(0.31 / 0.5 * 7))) + 7 * int(np.rint(0.2 / 0.5 * 7)) - 0
    assert q[0, 0] == want
    # non-linear device: ONE evaluation of the non-linearity per write, at the state the write finds
    v = 0.8
    cn = xo.make_config(flags=xo.PULSE_MAGNITUDE | xo.UPD_NL, upd_nl_v=v)
    g0, w_max = 0.25, 2.0
    Wn = xo.update_pulsed(cn, np.array([[g0 * w_max]], np.float32), np.array([[2.0], [-2.0]], np.float32),
                          np.array([[-0.5], [-0.25]], np.float32), w_max, 2.0, 0.5, 4, 2.0 ** -8)
    g1 = g0 + 16 * 2.0 ** -8 * np.exp(-np.float64(np.float32(v)) * 0.5 * (g0 + 1))                      # up by 4 x 4 quanta
    g2 = g1 - 8 * 2.0 ** -8 * np.exp(-np.float64(np.float32(v)) * (1 - 0.5 * (g1 + 1)))                 # down by 4 x 2
    assert Wn[0, 0] == np.float32(w_max * g2)
    # a time-coded write of the same size evaluates the non-linearity pulse by pulse: not the same number
    Wt = xo.update_pulsed(xo.make_config(flags=xo.PULSE_CODED | xo.UPD_NL, upd_nl_v=v), np.array([[g0 * w_max]], np.float32),
                          np.array([[2.0]], np.float32), np.array([[-0.5]], np.float32), w_max, 2.0, 0.5, 16, 2.0 ** -8)
    Wm = xo.update_pulsed(cn, np.array([[g0 * w_max]], np.float32), np.array([[2.0]], np.float32),
                          np.array([[-0.5]], np.float32), w_max, 2.0, 0.5, 4, 2.0 ** -8)
    assert Wt[0, 0] != Wm[0, 0] and abs(float(Wt[0, 0]) - float(Wm[0, 0])) < 1e-2
    # write noise: one draw per write (normal number m * 32 of the device's stream), standard deviation
    # gamma sqrt(lr quanta dw_min) with lr = bl^2 dw_min w_max / (x_range d_range)
    gam = 0.6
    cz = xo.make_config(flags=xo.PULSE_MAGNITUDE | xo.UPD_NOISE, upd_noise_gamma=gam, seed=21)
    Wz = xo.update_pulsed(cz, np.zeros((1, 1), np.float32), np.array([[0.0], [1.0]], np.float32), np.array([[0.3], [-0.25]], np.float32),
                          4.0, 2.0, 0.5, 6, dw, step=6)
    quanta_1 = 3 * 3
    lr_eq = 36 * dw * 4.0 / (2.0 * 0.5)
    g = quanta_1 * dw + np.float64(np.float32(gam)) * np.sqrt(lr_eq * dw) * np.sqrt(quanta_1) * xo.normal(21, 5, 6 << 31, 1 * 32)
    assert Wz[0, 0] == np.float32(4.0 * g)
    # time-coded and magnitude-coded pulses exclude each other
    with pytest.raises(AssertionError):
        xo.update_pulsed(xo.make_config(flags=xo.PULSE_MAGNITUDE | xo.PULSE_CODED), W0, X, D, 1.5, 2.0, 0.5, bl, dw)


def test_pair_update(xo):
    """Update with the two devices of a weight as states of their own."""
    rng = np.random.default_rng(5)
    M, K, N, w_max, lr = 9, 6, 7, 1.5, 0.05
    X = rng.standard_normal((M, K)).astype(np.float32)
    D = (rng.standard_normal((M, N)) * 0.1).astype(np.float32)
    W0 = rng.uniform(-0.8, 0.8, size=(K, N)).astype(np.float32)
    Gp0, Gn0 = xo.pair_init(W0, w_max)
    g = W0.astype(np.float64) / w_max
    assert np.array_equal(Gp0, (0.5 * (1 + g)).astype(np.float32)) and np.array_equal(Gn0, (0.5 * (1 - g)).astype(np.float32))
    # ideal devices: the pair's difference moves exactly as the one effective device of the aggregate model
    ideal = xo.make_config(flags=0)
    Gp, Gn, W1 = xo.update_pair(ideal, Gp0, Gn0, X, D, w_max, 1.0 / w_max, lr, step=2)
    assert np.array_equal(W1, (w_max * (Gp.astype(np.float64) - Gn)).astype(np.float32))            # W is the stored pair's difference
    assert np.abs(W1.astype(np.float64) - xo.update(ideal, W0, X, D, w_max, 1.0 / w_max, lr)).max() < 3e-7 * w_max
    grad = X.astype(np.float64).T @ D.astype(np.float64)
    assert np.allclose(Gp.astype(np.float64) - Gp0, -lr * 0.5 * grad / w_max, atol=1e-7)             # half the change each,
    assert np.allclose(Gn.astype(np.float64) - Gn0, +lr * 0.5 * grad / w_max, atol=1e-7)             # in opposite directions
    # every device clamps on its own
    gp = np.array([[0.99, 0.99, 0.5]], np.float32)
    gn = np.array([[0.01, 0.50, 0.02]], np.float32)
    x, d = np.array([[1.0]], np.float32), np.array([[-1.0, -1.0, 1.0]], np.float32)                 # delta = -1, -1, +1; lr 0.1
    Cp, Cn, Cw = xo.update_pair(ideal, gp, gn, x, d, 2.0, 1.0, 0.1)
    assert np.allclose(Cp, [[1.0, 1.0, 0.45]], atol=1e-7) and np.allclose(Cn, [[0.0, 0.45, 0.07]], atol=1e-7)
    assert np.allclose(Cw, 2.0 * (Cp.astype(np.float64) - Cn), atol=1e-6)
    assert Cp[0, 0] == 1.0 and Cn[0, 0] == 0.0
    # write non-linearity: each device at its own state and direction (rising exp(-v g), falling exp(-v (1 - g)))
    v = 0.7
    nl = xo.make_config(flags=xo.UPD_NL, upd_nl_v=v)
    vf = np.float64(np.float32(v))
    for delta in (0.4, -0.4):
        Np, Nn, _ = xo.update_pair(nl, np.array([[0.3]], np.float32), np.array([[0.6]], np.float32), np.array([[1.0]], np.float32),
                                   np.array([[delta]], np.float32), 1.0, 1.0, 0.5)
        half = 0.5 * np.float64(np.float32(delta))
        p0, n0 = np.float64(np.float32(0.3)), np.float64(np.float32(0.6))
        if delta > 0:      # weight falls: positive device falls, negative device rises
            want_p, want_n = p0 - 0.5 * half * np.exp(-vf * (1 - p0)), n0 + 0.5 * half * np.exp(-vf * n0)
        else:
            want_p, want_n = p0 - 0.5 * half * np.exp(-vf * p0), n0 + 0.5 * half * np.exp(-vf * (1 - n0))
        assert Np[0, 0] == np.float32(want_p) and Nn[0, 0] == np.float32(want_n)
    # mirror symmetry: swapping the two devices and the sign of the change swaps the results
    Ap, An, _ = xo.update_pair(nl, np.array([[0.3]], np.float32), np.array([[0.6]], np.float32), np.array([[1.0]], np.float32),
                               np.array([[0.4]], np.float32), 1.0, 1.0, 0.5)
    Bp, Bn, _ = xo.update_pair(nl, np.array([[0.6]], np.float32), np.array([[0.3]], np.float32), np.array([[1.0]], np.float32),
                               np.array([[-0.4]], np.float32), 1.0, 1.0, 0.5)
    assert Ap[0, 0] == Bn[0, 0] and An[0, 0] == Bp[0, 0]
    # write noise: a draw per device (numbers 2 i and 2 i + 1 of stream 6), sigma = gamma sqrt(|delta| / 2) each,
    # so the weight's noise variance is that of the effective device, gamma^2 |delta|
    gam, n_dev = 0.5, 40000
    nz = xo.make_config(flags=xo.UPD_NOISE, upd_noise_gamma=gam, seed=17)
    half_state = np.full((1, n_dev), 0.5, np.float32)
    delta = 0.02
    Zp, Zn, Zw = xo.update_pair(nz, half_state, half_state, np.array([[1.0]], np.float32), np.full((1, n_dev), delta, np.float32),
                                1.0, 1.0, 0.1, step=4)
    dp = Zp.astype(np.float64) - 0.5 + 0.1 * 0.5 * np.float64(np.float32(delta))
    dn = Zn.astype(np.float64) - 0.5 - 0.1 * 0.5 * np.float64(np.float32(delta))
    sigma = 0.1 * gam * np.sqrt(delta / 2)
    assert abs(dp.std() / sigma - 1) < 0.02 and abs(dn.std() / sigma - 1) < 0.02 and abs(dp.mean()) < 4 * sigma / np.sqrt(n_dev)
    assert abs(np.corrcoef(dp.ravel(), dn.ravel())[0, 1]) < 0.02
    assert abs((Zw.astype(np.float64)).std() / (0.1 * gam * np.sqrt(delta)) - 1) < 0.02
    want0 = 0.5 - 0.1 * (0.5 * np.float64(np.float32(delta)) + np.float64(np.float32(gam)) * np.sqrt(0.5 * np.float64(np.float32(delta))) * xo.normal(17, 6, 4, 0))
    want1 = 0.5 + 0.1 * (0.5 * np.float64(np.float32(delta)) + np.float64(np.float32(gam)) * np.sqrt(0.5 * np.float64(np.float32(delta))) * xo.normal(17, 6, 4, 2 * 3 + 1))
    assert Zp[0, 0] == np.float32(want0) and Zn[0, 3] == np.float32(want1)
