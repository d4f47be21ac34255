"""One training step of a CIFAR-style residual network (3 stages of n basic blocks, 6n + 2 weight
layers; n = 3 is ResNet-20) on emulated crossbars: every convolution and the classifier run through
the crossbar kernels (forward, backward, update: Sec. IV), everything else through the digital
peripheral kernels (Sec. IV-B).  This module only sequences calls of the C-ABI binding and keeps the
tensors a backward pass needs; it holds no arithmetic of its own.

Input ranges: every crossbar layer needs the range of its inputs (x_scale), of its errors (g_scale) and
of its weights (w_max).  They are data dependent (Sec. IV-B) and are fixed by `calibrate()` from one
batch: the observed maxima times a head-room factor.
"""
import math

import torch

from . import xbar as xb

HEADROOM_W, HEADROOM_X, HEADROOM_G = 2.0, 1.5, 4.0


class CrossbarLayer:
    """One weight layer: W[K][N], its conductance planes of the current step, its ranges."""

    def __init__(self, cfg_kwargs, K, N, geom, signed_input, gen, device):
        flags = cfg_kwargs["flags"] | (xb.INPUT_SIGNED if signed_input else 0)
        self.cfg = xb.make_config(**dict(cfg_kwargs, flags=flags))
        self.K, self.N, self.geom = K, N, geom
        self.W = torch.randn((K, N), generator=gen, device=device, dtype=torch.float32) * math.sqrt(2.0 / K)
        self.w_max = HEADROOM_W * xb.absmax(self.W)
        self.x_scale = self.g_scale = 1.0
        self.planes = torch.empty(xb.planes_bytes(self.cfg, K, N), dtype=torch.uint8, device=device)
        self.x = None

    def forward(self, x, step, ws):
        xb.tile(self.cfg, self.W, self.w_max, step, planes=self.planes)
        self.x = x
        if self.geom is None:
            return xb.fwd(self.cfg, self.planes, x, self.N, self.w_max, self.x_scale, ws=ws)
        return xb.conv_fwd(self.cfg, self.planes, x, self.geom, self.N, self.w_max, self.x_scale, ws=ws)

    def backward(self, dy, step, lr, ws, need_dx=True):
        """Error to the layer input through the same conductances, then the in-place write of W."""
        dx = None
        if self.geom is None:
            if need_dx:
                dx = xb.bwd(self.cfg, self.planes, dy, self.K, self.w_max, self.g_scale, ws=ws)
            xb.update(self.cfg, self.W, self.x, dy, self.w_max, 1.0 / self.w_max, lr, step, ws=ws)
        else:
            if need_dx:
                dx = xb.conv_bwd(self.cfg, self.planes, dy, self.geom, self.N, self.w_max, self.g_scale, ws=ws)
            xb.conv_update(self.cfg, self.W, self.x, dy, self.geom, self.w_max, 1.0 / self.w_max, lr, step, ws=ws)
        return dx

    def workspace_bytes(self, batch_rows):
        if self.geom is None:
            return max(xb.workspace_bytes(self.cfg, op, batch_rows, self.K, self.N) for op in (0, 1, 2))
        return max(xb.conv_workspace_bytes(self.cfg, op, self.geom, self.N) for op in (0, 1, 2))


class BatchNorm:
    def __init__(self, channels, device):
        self.gamma = torch.ones(channels, dtype=torch.float32, device=device)
        self.beta = torch.zeros(channels, dtype=torch.float32, device=device)
        self.saved = None

    def forward(self, x, ws):
        y, mean, invstd = xb.bn_fwd(x, self.gamma, self.beta, 1e-5, ws=ws)
        self.saved = (x, mean, invstd)
        return y

    def backward(self, dy, lr, ws):
        x, mean, invstd = self.saved
        dx, dgamma, dbeta = xb.bn_bwd(x, dy, self.gamma, mean, invstd, ws=ws)
        xb.sgd(self.gamma, dgamma, lr)
        xb.sgd(self.beta, dbeta, lr)
        return dx


class ResNetCifar:
    def __init__(self, cfg_kwargs, batch, n_blocks=3, image=32, classes=10, widths=(16, 32, 64), seed=0, device="cuda"):
        gen = torch.Generator(device=device)
        gen.manual_seed(seed)
        self.batch, self.image, self.classes = batch, image, classes
        conv = lambda hw, cin, cout, stride, signed: CrossbarLayer(
            cfg_kwargs, 9 * cin, cout, xb.conv_geom(batch, hw, hw, cin, 3, 3, stride, 1), signed, gen, device)
        self.stem, self.stem_bn = conv(image, 3, widths[0], 1, True), BatchNorm(widths[0], device)
        self.blocks = []
        cin, hw = widths[0], image
        for stage, width in enumerate(widths):
            for b in range(n_blocks):
                stride = 2 if (b == 0 and stage > 0) else 1
                hw_out = (hw + stride - 1) // stride
                self.blocks.append(dict(a=conv(hw, cin, width, stride, False), bn_a=BatchNorm(width, device),
                                        b=conv(hw_out, width, width, 1, False), bn_b=BatchNorm(width, device),
                                        stride=stride, cin=cin, width=width))
                cin, hw = width, hw_out
        self.fc = CrossbarLayer(cfg_kwargs, cin, classes, None, False, gen, device)
        self.layers = [self.stem] + [blk[k] for blk in self.blocks for k in ("a", "b")] + [self.fc]
        nbytes = max(max(L.workspace_bytes(batch) for L in self.layers),
                     xb.lib().xbar_bn_workspace_bytes(batch * image * image, max(widths)), 4096)
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.step_no = 0

    # ---- forward / backward ---------------------------------------------------------------------
    def forward(self, images, step):
        ws = self.ws
        a = xb.relu_fwd(self.stem_bn.forward(self.stem.forward(images, step, ws), ws))
        self.stem_out = a
        for blk in self.blocks:
            blk["in"] = a
            h = xb.relu_fwd(blk["bn_a"].forward(blk["a"].forward(a, step, ws), ws))
            blk["mid"] = h
            h = blk["bn_b"].forward(blk["b"].forward(h, step, ws), ws)
            skip = a if (blk["stride"] == 1 and blk["cin"] == blk["width"]) else xb.shortcut_fwd(a, blk["stride"], blk["width"])
            a = xb.relu_fwd(xb.add(h, skip))
            blk["out"] = a
        self.pooled = xb.avgpool_fwd(a)
        self.feat_shape = tuple(a.shape)
        return self.fc.forward(self.pooled, step, ws)

    def backward(self, dlogits, step, lr):
        ws = self.ws
        d = xb.avgpool_bwd(self.fc.backward(dlogits, step, lr, ws), self.feat_shape)
        for blk in reversed(self.blocks):
            d = xb.relu_bwd(blk["out"], d)                       # error of the sum: goes to both branches
            h = blk["b"].backward(blk["bn_b"].backward(d, lr, ws), step, lr, ws)
            h = blk["a"].backward(blk["bn_a"].backward(xb.relu_bwd(blk["mid"], h), lr, ws), step, lr, ws)
            if blk["stride"] == 1 and blk["cin"] == blk["width"]:
                d = xb.add(h, d)
            else:
                d = xb.add(h, xb.shortcut_bwd(d, tuple(blk["in"].shape), blk["stride"]))
        d = self.stem_bn.backward(xb.relu_bwd(self.stem_out, d), lr, ws)
        self.stem.backward(d, step, lr, ws, need_dx=False)

    def train_step(self, images, labels, lr):
        """One SGD step on a batch: returns the per-sample losses (device tensor)."""
        step = self.step_no
        logits = self.forward(images, step)
        loss, dlogits = xb.softmax_xent(logits, labels, 1.0 / images.shape[0])
        self.backward(dlogits, step, lr)
        self.step_no += 1
        return loss

    def calibrate(self, images, labels):
        calibrate_ranges(self, images, labels)

    def _bns(self):
        return [self.stem_bn] + [blk[k] for blk in self.blocks for k in ("bn_a", "bn_b")]


def calibrate_ranges(net, images, labels):
    """Fixes x_scale / g_scale of every crossbar layer of `net` from one batch: a pass with generous
    ranges records the maxima each layer sees, the ranges become those maxima times a head-room factor.
    No weight is changed."""
    seen_x, seen_g = {}, {}
    real_fwd, real_bwd = CrossbarLayer.forward, CrossbarLayer.backward

    def probe_fwd(layer, x, step, ws):
        seen_x[id(layer)] = xb.absmax(x)
        layer.x_scale = seen_x[id(layer)] or 1.0
        return real_fwd(layer, x, step, ws)

    def probe_bwd(layer, dy, step, lr, ws, need_dx=True):
        seen_g[id(layer)] = xb.absmax(dy)
        layer.g_scale = seen_g[id(layer)] or 1.0
        saved = layer.W.clone()
        out = real_bwd(layer, dy, step, 0.0, ws, need_dx)
        layer.W.copy_(saved)                                   # lr = 0 still rounds W through its range: undo
        return out

    bn_state = [(bn, bn.gamma.clone(), bn.beta.clone()) for bn in net._bns()]
    CrossbarLayer.forward, CrossbarLayer.backward = probe_fwd, probe_bwd
    try:
        logits = net.forward(images, 0)
        _, dlogits = xb.softmax_xent(logits, labels, 1.0 / images.shape[0])
        net.backward(dlogits, 0, 0.0)
    finally:
        CrossbarLayer.forward, CrossbarLayer.backward = real_fwd, real_bwd
    for bn, gamma, beta in bn_state:
        bn.gamma.copy_(gamma)
        bn.beta.copy_(beta)
    for layer in net.layers:
        layer.x_scale = HEADROOM_X * (seen_x[id(layer)] or 1.0)
        layer.g_scale = HEADROOM_G * (seen_g[id(layer)] or 1.0)
