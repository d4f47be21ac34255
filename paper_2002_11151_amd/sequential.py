"""One training step of a plain feed-forward stack (convolutions, ReLU, max pooling, fully connected
layers: VGG-16, multi-layer perceptrons) on emulated crossbars: weight layers through the crossbar
kernels (Sec. IV), the rest through the digital peripheral kernels (Sec. IV-B).  Only sequences calls of
the C-ABI binding.

A network is a list of layer specs:
    ("conv", out_channels, kernel, stride, pad) | ("relu",) | ("sigmoid",) | ("maxpool", kernel, stride) |
    ("flatten",) | ("fc", out_features)
"""
import torch

from . import xbar as xb
from .resnet_cifar import CrossbarLayer, Network


def vgg16_spec(classes=1000):
    spec = []
    for width, n in ((64, 2), (128, 2), (256, 3), (512, 3), (512, 3)):
        for _ in range(n):
            spec += [("conv", width, 3, 1, 1), ("relu",)]
        spec.append(("maxpool", 2, 2))
    return spec + [("flatten",), ("fc", 4096), ("relu",), ("fc", 4096), ("relu",), ("fc", classes)]


def mlp_spec(hidden=(500,), classes=10, activation="relu"):
    spec = [("flatten",)]
    for h in hidden:
        spec += [("fc", h), (activation,)]
    return spec + [("fc", classes)]


class Sequential(Network):
    def __init__(self, cfg_kwargs, spec, batch, in_shape, signed_input=True, seed=0, device="cuda"):
        """in_shape: (height, width, channels) of one sample, or (features,)."""
        gen = torch.Generator(device=device)
        gen.manual_seed(seed)
        self.batch, self.stack, self.layers = batch, [], []
        shape = tuple(in_shape)
        signed = signed_input
        for op in spec:
            kind = op[0]
            if kind == "conv":
                _, cout, k, stride, pad = op
                h, w, c = shape
                geom = xb.conv_geom(batch, h, w, c, k, k, stride, pad)
                layer = CrossbarLayer(self, cfg_kwargs, k * k * c, cout, geom, signed, gen, device)
                self.stack.append(("layer", layer))
                self.layers.append(layer)
                shape, signed = (geom.out_h, geom.out_w, cout), True      # a raw layer output is signed
            elif kind == "fc":
                (features,) = shape
                layer = CrossbarLayer(self, cfg_kwargs, features, op[1], None, signed, gen, device)
                self.stack.append(("layer", layer))
                self.layers.append(layer)
                shape, signed = (op[1],), True
            elif kind in ("relu", "sigmoid"):
                self.stack.append((kind, None))
                signed = False                                            # both outputs are non-negative
            elif kind == "maxpool":
                h, w, c = shape
                geom = xb.conv_geom(batch, h, w, c, op[1], op[1], op[2], 0)
                self.stack.append(("maxpool", geom))
                shape = (geom.out_h, geom.out_w, c)
            elif kind == "flatten":
                n = 1
                for d in shape:
                    n *= d
                self.stack.append(("flatten", shape))
                shape = (n,)
            else:
                raise ValueError("unknown layer spec %r" % (op,))
        self.ws = torch.empty(max(max(L.workspace_bytes(batch) for L in self.layers), 4096), dtype=torch.uint8,
                              device=device)
        self.saved = [None] * len(self.stack)
        self.step_no = 0

    def forward(self, x, step):
        for i, (kind, arg) in enumerate(self.stack):
            if kind == "layer":
                x = arg.forward(x, step, self.ws)
            elif kind == "relu":
                x = self.ops.relu_fwd(x)
                self.saved[i] = x
            elif kind == "sigmoid":
                x = self.ops.sigmoid_fwd(x)
                self.saved[i] = x
            elif kind == "maxpool":
                x, self.saved[i] = self.ops.maxpool_fwd(x, arg)
            else:                                             # flatten: NHWC rows are already contiguous
                self.saved[i] = tuple(x.shape)
                x = x.reshape(x.shape[0], -1)
        return x

    def backward(self, d, step, lr):
        first_layer = next(i for i, (kind, _) in enumerate(self.stack) if kind == "layer")
        for i in range(len(self.stack) - 1, -1, -1):
            kind, arg = self.stack[i]
            if kind == "layer":
                d = arg.backward(d, step, lr, self.ws, need_dx=i != first_layer)
            elif kind == "relu":
                d = self.ops.relu_bwd(self.saved[i], d)
            elif kind == "sigmoid":
                d = self.ops.sigmoid_bwd(self.saved[i], d)
            elif kind == "maxpool":
                d = self.ops.maxpool_bwd(d, self.saved[i], arg)
            else:
                d = d.reshape(self.saved[i])
            if d is None:
                break
