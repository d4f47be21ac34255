"""TEST INFRASTRUCTURE: convolution layers on top of the oracle's matrix operations (Sec. IV: the
kernels of a layer are unrolled into the columns of the crossbar weight matrix; every output position
applies its input patch to the rows).

Plain definitions: `im2col` writes the patch of every output position as one row, `col2im` is its
adjoint (every input pixel adds up the entries of all patches that contain it).  Activations are NHWC,
the patch index is (kh, kw, c) with c fastest, positions outside the image are 0.
"""
import numpy as np


def out_size(n, k, stride, pad):
    return (n + 2 * pad - k) // stride + 1


def im2col(X, k_h, k_w, stride, pad):
    """X[B][H][W][C] -> patches[B * OH * OW][k_h * k_w * C]."""
    B, H, W, C = X.shape
    OH, OW = out_size(H, k_h, stride, pad), out_size(W, k_w, stride, pad)
    out = np.zeros((B, OH, OW, k_h, k_w, C), dtype=X.dtype)
    for oh in range(OH):
        for ow in range(OW):
            for kh in range(k_h):
                for kw in range(k_w):
                    ih, iw = oh * stride - pad + kh, ow * stride - pad + kw
                    if 0 <= ih < H and 0 <= iw < W:
                        out[:, oh, ow, kh, kw, :] = X[:, ih, iw, :]
    return out.reshape(B * OH * OW, k_h * k_w * C)


def col2im(cols, shape, k_h, k_w, stride, pad):
    """Adjoint of im2col: cols[B * OH * OW][k_h * k_w * C] -> float64 sums in the NHWC `shape`."""
    B, H, W, C = shape
    OH, OW = out_size(H, k_h, stride, pad), out_size(W, k_w, stride, pad)
    cols = np.asarray(cols, dtype=np.float64).reshape(B, OH, OW, k_h, k_w, C)
    out = np.zeros(shape, dtype=np.float64)
    for oh in range(OH):
        for ow in range(OW):
            for kh in range(k_h):
                for kw in range(k_w):
                    ih, iw = oh * stride - pad + kh, ow * stride - pad + kw
                    if 0 <= ih < H and 0 <= iw < W:
                        out[:, ih, iw, :] += cols[:, oh, ow, kh, kw, :]
    return out
