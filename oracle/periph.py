"""TEST INFRASTRUCTURE: the digital peripheral operations (Sec. IV-B: ReLU, batch normalisation and
pooling are computed digitally), the softmax cross-entropy loss and plain SGD, written out from their
textbook definitions in float64 numpy.  NHWC tensors, channels last."""
import numpy as np


def relu_fwd(x):
    return np.maximum(np.asarray(x, dtype=np.float64), 0.0)


def relu_bwd(y, dy):
    return np.where(np.asarray(y) > 0, np.asarray(dy, dtype=np.float64), 0.0)


def sigmoid_fwd(x):
    """Logistic function 1 / (1 + exp(-x)) (Sec. IV-B lists it with the digital peripherals)."""
    return 1.0 / (1.0 + np.exp(-np.asarray(x, dtype=np.float64)))


def sigmoid_bwd(y, dy):
    """From the forward output: dx = dy y (1 - y)."""
    y = np.asarray(y, dtype=np.float64)
    return np.asarray(dy, dtype=np.float64) * y * (1.0 - y)


def bn_fwd(x, gamma, beta, eps):
    """Training-mode batch normalisation over all axes but the last: returns y, mean, invstd."""
    x = np.asarray(x, dtype=np.float64)
    flat = x.reshape(-1, x.shape[-1])
    mean = flat.mean(axis=0)
    var = ((flat - mean) ** 2).mean(axis=0)              # biased
    invstd = 1.0 / np.sqrt(var + eps)
    y = np.asarray(gamma, dtype=np.float64) * (x - mean) * invstd + np.asarray(beta, dtype=np.float64)
    return y, mean, invstd


def bn_bwd(x, dy, gamma, mean, invstd):
    """Gradient of bn_fwd through the batch statistics: returns dx, dgamma, dbeta."""
    x, dy = np.asarray(x, dtype=np.float64), np.asarray(dy, dtype=np.float64)
    rows = x.size // x.shape[-1]
    xhat = (x - mean) * invstd
    axes = tuple(range(x.ndim - 1))
    dbeta = dy.sum(axis=axes)
    dgamma = (dy * xhat).sum(axis=axes)
    dx = np.asarray(gamma, dtype=np.float64) * invstd * (dy - dbeta / rows - xhat * dgamma / rows)
    return dx, dgamma, dbeta


def avgpool_fwd(x):
    x = np.asarray(x, dtype=np.float64)
    return x.reshape(x.shape[0], -1, x.shape[-1]).mean(axis=1)


def avgpool_bwd(dy, shape):
    positions = int(np.prod(shape[1:-1]))
    dy = np.asarray(dy, dtype=np.float64)
    return np.broadcast_to(dy.reshape(shape[0], *([1] * (len(shape) - 2)), shape[-1]) / positions, shape).copy()


def maxpool_fwd(x, k, stride, pad):
    """Returns y[B][OH][OW][C] and argmax (ih * W + iw of the first maximum in scan order)."""
    x = np.asarray(x, dtype=np.float64)
    B, H, W, C = x.shape
    OH, OW = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    y = np.full((B, OH, OW, C), -np.inf)
    arg = np.full((B, OH, OW, C), -1, dtype=np.int32)
    for oh in range(OH):
        for ow in range(OW):
            for kh in range(k):
                for kw in range(k):
                    ih, iw = oh * stride - pad + kh, ow * stride - pad + kw
                    if 0 <= ih < H and 0 <= iw < W:
                        v = x[:, ih, iw, :]
                        better = v > y[:, oh, ow, :]
                        y[:, oh, ow, :] = np.where(better, v, y[:, oh, ow, :])
                        arg[:, oh, ow, :] = np.where(better, ih * W + iw, arg[:, oh, ow, :])
    return y, arg


def maxpool_bwd(dy, arg, shape):
    B, H, W, C = shape
    dx = np.zeros((B, H * W, C))
    dy = np.asarray(dy, dtype=np.float64)
    OH, OW = arg.shape[1:3]
    for oh in range(OH):
        for ow in range(OW):
            for b in range(B):
                for c in range(C):
                    dx[b, arg[b, oh, ow, c], c] += dy[b, oh, ow, c]
    return dx.reshape(shape)


def softmax_xent(logits, labels, scale):
    """Per-sample loss -log softmax[label] and dlogits = scale * (softmax - onehot)."""
    z = np.asarray(logits, dtype=np.float64)
    z = z - z.max(axis=1, keepdims=True)
    p = np.exp(z) / np.exp(z).sum(axis=1, keepdims=True)
    idx = np.arange(z.shape[0])
    loss = -np.log(p[idx, labels])
    d = p.copy()
    d[idx, labels] -= 1.0
    return loss, scale * d


def shortcut_fwd(x, stride, out_channels):
    """Parameter-free residual shortcut: subsample the positions, add zero channels (half in front)."""
    x = np.asarray(x, dtype=np.float64)[:, ::stride, ::stride, :]
    lo = (out_channels - x.shape[-1]) // 2
    y = np.zeros(x.shape[:-1] + (out_channels,))
    y[..., lo:lo + x.shape[-1]] = x
    return y


def shortcut_bwd(dy, shape, stride):
    dy = np.asarray(dy, dtype=np.float64)
    lo = (dy.shape[-1] - shape[-1]) // 2
    dx = np.zeros(shape)
    dx[:, ::stride, ::stride, :] = dy[..., lo:lo + shape[-1]]
    return dx
