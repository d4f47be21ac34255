"""One training step of an ImageNet-style bottleneck residual network (7x7 stem, 3x3 max pool, stages
of [1x1, 3x3, 1x1] blocks with the stride on the 3x3 convolution and a 1x1 projection on the shortcut
of every first block, global average pool, classifier; blocks (3, 4, 6, 3) and widths (64, 128, 256,
512) give ResNet-50) on emulated crossbars: every convolution and the classifier run through the
crossbar kernels (Sec. IV), everything else through the digital peripheral kernels (Sec. IV-B).  Like
its CIFAR-size sibling this module only sequences calls of the C-ABI binding.
"""
import torch

from . import xbar as xb
from .resnet_cifar import BatchNorm, CrossbarLayer, Network


class ResNetBottleneck(Network):
    def __init__(self, cfg_kwargs, batch, image=224, classes=1000, blocks=(3, 4, 6, 3), widths=(64, 128, 256, 512),
                 stem=64, seed=0, device="cuda"):
        gen = torch.Generator(device=device)
        gen.manual_seed(seed)
        self.batch = batch

        def conv(hw, cin, cout, k, stride, pad, signed=False):
            return CrossbarLayer(self, cfg_kwargs, k * k * cin, cout, xb.conv_geom(batch, hw, hw, cin, k, k, stride, pad),
                                 signed, gen, device)

        self.stem, self.stem_bn = conv(image, 3, stem, 7, 2, 3, True), BatchNorm(self, stem, device)
        hw = (image + 6 - 7) // 2 + 1
        self.pool_geom = xb.conv_geom(batch, hw, hw, stem, 3, 3, 2, 1)
        hw = self.pool_geom.out_h
        self.blocks = []
        cin = stem
        for stage, (width, n) in enumerate(zip(widths, blocks)):
            for b in range(n):
                stride = 2 if (b == 0 and stage > 0) else 1
                hw_out = (hw + 2 - 3) // stride + 1
                blk = dict(a=conv(hw, cin, width, 1, 1, 0), bn_a=BatchNorm(self, width, device),
                           b=conv(hw, width, width, 3, stride, 1), bn_b=BatchNorm(self, width, device),
                           c=conv(hw_out, width, 4 * width, 1, 1, 0), bn_c=BatchNorm(self, 4 * width, device))
                if b == 0:                              # projection shortcut (changes width and, later, size)
                    blk["down"], blk["bn_down"] = conv(hw, cin, 4 * width, 1, stride, 0), BatchNorm(self, 4 * width, device)
                self.blocks.append(blk)
                cin, hw = 4 * width, hw_out
        self.fc = CrossbarLayer(self, cfg_kwargs, cin, classes, None, False, gen, device)
        self.layers = [self.stem] + [blk[k] for blk in self.blocks for k in ("a", "b", "c", "down") if k in blk] + [self.fc]
        rows = batch * ((image + 6 - 7) // 2 + 1) ** 2
        nbytes = max(max(L.workspace_bytes(batch) for L in self.layers),
                     xb.lib().xbar_bn_workspace_bytes(rows, max(stem, 4 * max(widths))), 4096)
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.step_no = 0

    def forward(self, images, step):
        ws, ops = self.ws, self.ops
        a = ops.relu_fwd(self.stem_bn.forward(self.stem.forward(images, step, ws), ws))
        self.stem_out = a
        a, self.pool_arg = ops.maxpool_fwd(a, self.pool_geom)
        for blk in self.blocks:
            h = ops.relu_fwd(blk["bn_a"].forward(blk["a"].forward(a, step, ws), ws))
            blk["act_a"] = h
            h = ops.relu_fwd(blk["bn_b"].forward(blk["b"].forward(h, step, ws), ws))
            blk["act_b"] = h
            h = blk["bn_c"].forward(blk["c"].forward(h, step, ws), ws)
            skip = blk["bn_down"].forward(blk["down"].forward(a, step, ws), ws) if "down" in blk else a
            a = ops.relu_fwd(ops.add(h, skip))
            blk["out"] = a
        self.pooled = ops.avgpool_fwd(a)
        self.feat_shape = tuple(a.shape)
        return self.fc.forward(self.pooled, step, ws)

    def backward(self, dlogits, step, lr):
        ws, ops = self.ws, self.ops
        d = ops.avgpool_bwd(self.fc.backward(dlogits, step, lr, ws), self.feat_shape)
        for blk in reversed(self.blocks):
            d = ops.relu_bwd(blk["out"], d)                       # error of the sum: goes to both branches
            h = blk["c"].backward(blk["bn_c"].backward(d, lr, ws), step, lr, ws)
            h = blk["b"].backward(blk["bn_b"].backward(ops.relu_bwd(blk["act_b"], h), lr, ws), step, lr, ws)
            h = blk["a"].backward(blk["bn_a"].backward(ops.relu_bwd(blk["act_a"], h), lr, ws), step, lr, ws)
            if "down" in blk:
                d = blk["down"].backward(blk["bn_down"].backward(d, lr, ws), step, lr, ws)
            d = ops.add(h, d)
        d = ops.maxpool_bwd(d, self.pool_arg, self.pool_geom)
        d = self.stem_bn.backward(ops.relu_bwd(self.stem_out, d), lr, ws)
        self.stem.backward(d, step, lr, ws, need_dx=False)
