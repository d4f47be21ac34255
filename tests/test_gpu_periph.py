"""GPU parity of the digital peripheral kernels (through the C ABI) against their plain definitions."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def xb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2002_11151_amd import xbar
    xbar.lib()
    return xbar


def dev(a, dtype=np.float32):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=dtype)).cuda()


def close(got, want, tol=2e-6):
    got, want = got.cpu().numpy().astype(np.float64), np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape
    assert np.abs(got - want).max() <= tol * max(1.0, np.abs(want).max())


@pytest.mark.parametrize("B,H,W,C", [(3, 6, 5, 7), (4, 16, 16, 64), (2, 33, 17, 130), (128, 1, 1, 10)])
def test_batchnorm_relu_add(xb, B, H, W, C):
    from oracle import periph
    rng = np.random.default_rng(B + C)
    x = (rng.normal(size=(B, H, W, C)) * 2 + 0.5).astype(np.float32)
    dy = rng.normal(size=(B, H, W, C)).astype(np.float32)
    gamma, beta = rng.uniform(0.5, 1.5, size=C).astype(np.float32), rng.normal(size=C).astype(np.float32)
    y, mean, invstd = xb.bn_fwd(dev(x), dev(gamma), dev(beta), 1e-5)
    yo, mo, io = periph.bn_fwd(x, gamma, beta, 1e-5)
    close(y, yo)
    close(mean, mo)
    close(invstd, io)
    dx, dgamma, dbeta = xb.bn_bwd(dev(x), dev(dy), dev(gamma), mean, invstd)
    dxo, dgo, dbo = periph.bn_bwd(x, dy, gamma, mean.cpu().numpy().astype(np.float64), invstd.cpu().numpy().astype(np.float64))
    close(dx, dxo, 1e-5)
    close(dgamma, dgo, 1e-5)
    close(dbeta, dbo, 1e-5)
    r = xb.relu_fwd(dev(x))
    assert np.array_equal(r.cpu().numpy(), periph.relu_fwd(x).astype(np.float32))
    assert np.array_equal(xb.relu_bwd(r, dev(dy)).cpu().numpy(), periph.relu_bwd(r.cpu().numpy(), dy).astype(np.float32))
    s = xb.sigmoid_fwd(dev(x))
    assert np.abs(s.cpu().numpy() - periph.sigmoid_fwd(x)).max() <= 6e-8                  # half a unit in the last place below 1
    assert np.abs(xb.sigmoid_bwd(s, dev(dy)).cpu().numpy() - periph.sigmoid_bwd(s.cpu().numpy(), dy)).max() <= 1e-7 * np.abs(dy).max()
    assert np.array_equal(xb.add(dev(x), dev(dy)).cpu().numpy(), x + dy)
    p = dev(x.copy())
    xb.sgd(p, dev(dy), 0.1)
    close(p, x.astype(np.float64) - np.float32(0.1).astype(np.float64) * dy, 1e-6)


@pytest.mark.parametrize("B,H,W,C,k,stride,pad", [(2, 9, 8, 5, 3, 2, 1), (3, 8, 8, 64, 2, 2, 0), (1, 7, 7, 3, 3, 1, 1)])
def test_pooling(xb, B, H, W, C, k, stride, pad):
    from oracle import periph
    rng = np.random.default_rng(H + C)
    x = rng.normal(size=(B, H, W, C)).astype(np.float32)
    geom = xb.conv_geom(B, H, W, C, k, k, stride, pad)
    y, arg = xb.maxpool_fwd(dev(x), geom)
    yo, ao = periph.maxpool_fwd(x, k, stride, pad)
    assert np.array_equal(y.cpu().numpy(), yo.astype(np.float32))
    assert np.array_equal(arg.cpu().numpy(), ao)
    d = rng.normal(size=yo.shape).astype(np.float32)
    close(xb.maxpool_bwd(dev(d), arg, geom), periph.maxpool_bwd(d, ao, x.shape))
    a = xb.avgpool_fwd(dev(x))
    close(a, periph.avgpool_fwd(x))
    dg = rng.normal(size=(B, C)).astype(np.float32)
    close(xb.avgpool_bwd(dev(dg), x.shape), periph.avgpool_bwd(dg, x.shape))


@pytest.mark.parametrize("B,classes", [(5, 10), (64, 1000), (3, 1)])
def test_softmax_cross_entropy(xb, B, classes):
    from oracle import periph
    rng = np.random.default_rng(classes)
    z = (rng.normal(size=(B, classes)) * 4).astype(np.float32)
    labels = rng.integers(0, classes, size=B).astype(np.int32)
    loss, dz = xb.softmax_xent(dev(z), dev(labels, np.int32), 1.0 / B)
    lo, dzo = periph.softmax_xent(z, labels, np.float32(1.0 / B).astype(np.float64))
    close(loss, lo, 1e-6)
    close(dz, dzo, 1e-6)
    bad = labels.copy()
    bad[0] = classes                                          # unknown class: NaN loss, no fault
    loss, _ = xb.softmax_xent(dev(z), dev(bad, np.int32), 1.0)
    assert np.isnan(loss.cpu().numpy()[0]) and not np.isnan(loss.cpu().numpy()[1:]).any()
