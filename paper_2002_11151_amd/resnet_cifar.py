"""One training step of a CIFAR-style residual network (3 stages of n basic blocks, 6n + 2 weight
layers; n = 3 is ResNet-20) on emulated crossbars: every convolution and the classifier run through
the crossbar kernels (forward, backward, update: Sec. IV), everything else through the digital
peripheral kernels (Sec. IV-B).  This module only sequences calls of the C-ABI binding and keeps the
tensors a backward pass needs; it holds no arithmetic of its own.

Input ranges: every crossbar layer needs the range of its inputs (x_scale), of its errors (g_scale) and
of its weights (w_max).  They are data dependent (Sec. IV-B) and are fixed by `calibrate()` from one
batch: the observed maxima times a head-room factor.  The converter ranges (the maximum current through
the ADCs, which Sec. IV-B takes from output distribution statistics) can be fixed the same way: with
`calibrate(..., adc_quantile=q)` a second pass histograms the column currents of every layer on the device
and sets each range to the smallest power of two that holds the fraction q of them.
"""
import math

import torch

from . import xbar as xb

HEADROOM_W, HEADROOM_X, HEADROOM_G = 2.0, 1.5, 4.0


class CrossbarLayer:
    """One weight layer: W[K][N], its conductance planes of the current step, its ranges."""

    def __init__(self, net, cfg_kwargs, K, N, geom, signed_input, gen, device):
        self.net = net                 # supplies `ops` (the binding, or a stand-in that records / times its calls)
        flags = cfg_kwargs["flags"] | (xb.INPUT_SIGNED if signed_input else 0)
        # every layer keys its own random streams (device variation, write noise, pulse trains): layers of equal
        # shape must not see the same draws at the same step
        self.index = getattr(net, "n_crossbar_layers", 0)
        net.n_crossbar_layers = self.index + 1
        seed = (int(cfg_kwargs.get("seed", 0)) << 20) + self.index
        self.cfg = xb.make_config(**dict(cfg_kwargs, flags=flags, seed=seed))
        self.K, self.N, self.geom = K, N, geom
        self.W = torch.randn((K, N), generator=gen, device=device, dtype=torch.float32) * math.sqrt(2.0 / K)
        self.w_max = HEADROOM_W * net.ops.absmax(self.W)
        self.x_scale = self.g_scale = 1.0
        self.planes = torch.empty(xb.planes_bytes(self.cfg, K, N), dtype=torch.uint8, device=device)
        self.x = None
        self.profile = None                # stored wire distortion (with the profile flag), refreshed by forward()
        self.pair = None                   # (Gp, Gn) once the network updates the two devices of a weight separately
        self.seen_x = self.seen_g = None   # set while the ranges are being calibrated

    def forward(self, x, step, ws):
        ops = self.net.ops
        if self.net.calibrating and self.net.adc_quantile is None:
            self.seen_x = self.x_scale = ops.absmax(x) or 1.0
        if self.cfg.flags & xb.NI_WIRE_PROFILE:
            # the circuit-level model every `fcm_every` steps, its stored distortion profile in between (Sec. IV-D)
            if self.profile is None or step % self.net.fcm_every == 0:
                self.profile = ops.fcm_profile(self.cfg, self.W, self.w_max, step, ws=ws, profile=self.profile)
            ops.tile(self.cfg, self.W, self.w_max, step, self.profile, planes=self.planes)
        else:
            ops.tile(self.cfg, self.W, self.w_max, step, planes=self.planes)
        self.x = x
        if self.net.adc_quantile is not None:
            self.cfg.adc_fs_fwd = self._measured_range(xb.OP_FWD, x, self.x_scale, self.cfg.xbar_rows, ws)
        if self.geom is None:
            return ops.fwd(self.cfg, self.planes, x, self.N, self.w_max, self.x_scale, ws=ws)
        return ops.conv_fwd(self.cfg, self.planes, x, self.geom, self.N, self.w_max, self.x_scale, ws=ws)

    def backward(self, dy, step, lr, ws, need_dx=True):
        """Error to the layer input through the same conductances, then the in-place write of W (skipped
        while the ranges are being calibrated)."""
        ops = self.net.ops
        if self.net.calibrating and self.net.adc_quantile is None:
            self.seen_g = self.g_scale = ops.absmax(dy) or 1.0
        if self.net.adc_quantile is not None:
            self.cfg.adc_fs_bwd = self._measured_range(xb.OP_BWD, dy, self.g_scale, self.cfg.xbar_cols, ws)
        dx = None
        pulse = self.net.pulse
        if self.geom is None:
            if need_dx:
                dx = ops.bwd(self.cfg, self.planes, dy, self.K, self.w_max, self.g_scale, ws=ws)
            if not self.net.calibrating and pulse is None and self.net.pair_devices:
                ops.update_pair(self.cfg, *self._pair(), self.W, self.x, dy, self.w_max, 1.0 / self.w_max, lr, step, ws=ws)
            elif not self.net.calibrating and pulse is None:
                ops.update(self.cfg, self.W, self.x, dy, self.w_max, 1.0 / self.w_max, lr, step, ws=ws)
            elif not self.net.calibrating:
                # inputs fire in proportion to their size over the calibrated range; the error range then follows
                # from the learning rate: mean change = lr x dy / w_max  <=>  x_range d_range = bl dw_min w_max / lr
                bl, dw_min, d_range = self._pulse_ranges(pulse, lr)
                ops.update_pulsed(self.cfg, self.W, self.x, dy, self.w_max, self.x_scale, d_range, bl, dw_min, step, ws=ws)
        else:
            if need_dx:
                dx = ops.conv_bwd(self.cfg, self.planes, dy, self.geom, self.N, self.w_max, self.g_scale, ws=ws)
            if not self.net.calibrating and pulse is None and self.net.pair_devices:
                ops.conv_update_pair(self.cfg, *self._pair(), self.W, self.x, dy, self.geom, self.w_max, 1.0 / self.w_max, lr,
                                     step, ws=ws)
            elif not self.net.calibrating and pulse is None:
                ops.conv_update(self.cfg, self.W, self.x, dy, self.geom, self.w_max, 1.0 / self.w_max, lr, step, ws=ws)
            elif not self.net.calibrating:     # every output position is one sample of the pulse scheme
                bl, dw_min, d_range = self._pulse_ranges(pulse, lr)
                ops.conv_update_pulsed(self.cfg, self.W, self.x, dy, self.geom, self.w_max, self.x_scale, d_range, bl,
                                       dw_min, step, ws=ws)
        return dx

    def _pair(self):
        """The two device states of every weight (first use: placed symmetrically about mid-range)."""
        if self.pair is None:
            self.pair = self.net.ops.pair_init(self.W, self.w_max)
        return self.pair

    def _pulse_ranges(self, pulse, lr):
        """(bl, dw_min, d_range) of a pulse-level update whose mean is the update at learning rate lr:
        lr = slots dw_min w_max / (x_range d_range) with x_range = the calibrated input range.  Stochastic
        trains round without bias, so the pulse size is free and the error range follows from it; deterministic
        codes (in time or in magnitude) drop what is below half a level, so there the errors use their calibrated
        range and the pulse size follows."""
        bl, slots = pulse["bl"], self.net.ops.pulse_slots(self.cfg, pulse["bl"])
        if self.cfg.flags & (xb.PULSE_CODED | xb.PULSE_MAGNITUDE):
            return bl, lr * self.x_scale * self.g_scale / (slots * self.w_max), self.g_scale
        return bl, pulse["dw_min"], slots * pulse["dw_min"] * self.w_max / (lr * self.x_scale)

    def _measured_range(self, op, inp, in_scale, driven_lines, ws):
        """Converter range of one pass from the currents this input causes (statistics pass of the library)."""
        ops, cfg = self.net.ops, self.cfg
        # bins over everything a tile can carry: all driven lines at the top input level into full-level devices
        # (twice that for a single array with its off-state current)
        top = driven_lines * ((1 << cfg.stream_bits) - 1) * ((1 << cfg.slice_bits) - 1) * (2 if cfg.flags & xb.ADC_PER_ARRAY else 1)
        bin_width = top / (xb.ADC_HIST_BINS - 1.0)
        if self.geom is None:
            hist = ops.adc_histogram(cfg, self.planes, inp, self.K, self.N, in_scale, op, bin_width, ws=ws)
        else:
            hist = ops.conv_adc_histogram(cfg, self.planes, inp, self.geom, self.N, in_scale, op, bin_width, ws=ws)
        return ops.adc_range_from_histogram(hist, bin_width, self.net.adc_quantile)

    def workspace_bytes(self, batch_rows):
        fcm = xb.workspace_bytes(self.cfg, xb.OP_FCM, 1, self.K, self.N) if self.cfg.flags & xb.NI_WIRE_PROFILE else 0
        if self.geom is None:
            return max(fcm, *(xb.workspace_bytes(self.cfg, op, batch_rows, self.K, self.N)
                              for op in (xb.OP_FWD, xb.OP_BWD, xb.OP_UPDATE, xb.OP_UPDATE_PULSED)))
        return max(fcm, *(xb.conv_workspace_bytes(self.cfg, op, self.geom, self.N) for op in (xb.OP_FWD, xb.OP_BWD, xb.OP_UPDATE, xb.OP_UPDATE_PULSED)))


class BatchNorm:
    def __init__(self, net, channels, device):
        self.net = net
        self.gamma = torch.ones(channels, dtype=torch.float32, device=device)
        self.beta = torch.zeros(channels, dtype=torch.float32, device=device)
        self.saved = None

    def forward(self, x, ws):
        y, mean, invstd = self.net.ops.bn_fwd(x, self.gamma, self.beta, 1e-5, ws=ws)
        self.saved = (x, mean, invstd)
        return y

    def backward(self, dy, lr, ws):
        x, mean, invstd = self.saved
        ops = self.net.ops
        dx, dgamma, dbeta = ops.bn_bwd(x, dy, self.gamma, mean, invstd, ws=ws)
        if not self.net.calibrating:
            ops.sgd(self.gamma, dgamma, lr)
            ops.sgd(self.beta, dbeta, lr)
        return dx


class Network:
    """What the networks share: the binding they call (`ops`, replaceable by an object with the same
    functions that records or times the calls), the training step, the range calibration and the kind of
    weight update (aggregate write, or pulse by pulse when `pulse` is set).
    Subclasses provide forward(x, step), backward(dlogits, step, lr) and self.layers."""
    ops = xb
    calibrating = False
    fcm_every = 1         # with the stored-profile wire model: steps between two runs of the circuit-level model
    adc_quantile = None   # set while the converter ranges are being measured
    pulse = None     # dict(bl=slots per train, dw_min=state change per pulse): pulse-level updates of the crossbar layers
    pair_devices = False   # aggregate updates keep the positive and the negative device of a weight as states of their own

    def train_step(self, x, labels, lr):
        """One SGD step on a batch: returns the per-sample losses (device tensor)."""
        step = self.step_no
        logits = self.forward(x, step)
        loss, dlogits = self.ops.softmax_xent(logits, labels, 1.0 / x.shape[0])
        self.backward(dlogits, step, lr)
        self.step_no += 1
        return loss

    # ---- a training step as a HIP graph -----------------------------------------------------------
    def capture(self, x, labels, lr):
        """Captures one training step (fixed batch shape and learning rate) into a HIP graph: the step then costs one
        graph launch instead of several hundred kernel launches, which is what bounds the small networks.  The
        kernels' arguments are frozen in a graph, so the step number that keys the device variation and the write
        noise comes from a counter in device memory that the graph itself advances.  Runs one real step (the
        warm-up of the capture) and returns its losses; every `replay(x, labels)` is the next step."""
        # The circuit-level model runs when step % fcm_every == 0, a test the host makes per step: a graph would
        # freeze its outcome at capture time (a refresh on every replay, or on none).
        if self.fcm_every > 1 and any(L.cfg.flags & xb.NI_WIRE_PROFILE for L in self.layers):
            raise ValueError("capture(): the stored-profile wire model with fcm_every > 1 refreshes its profile on some "
                             "steps only, which a captured graph cannot express; run those steps eagerly")
        self._graph_x, self._graph_labels = x.clone(), labels.clone()
        self._graph_counter = torch.full((1,), self.step_no, dtype=torch.int64, device=x.device)
        main, side = torch.cuda.current_stream(), torch.cuda.Stream()
        side.wait_stream(main)
        xb.set_step_source(self._graph_counter)
        try:
            with torch.cuda.stream(side):
                first = self._counted_step(lr).clone()
            main.wait_stream(side)
            self._graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(self._graph, stream=side):
                self._graph_loss = self._counted_step(lr)
        finally:
            xb.set_step_source(None)
        self.step_no += 1
        return first

    def replay(self, x, labels):
        """The next training step from the captured graph; returns the per-sample losses (a buffer that the next
        replay overwrites)."""
        self._graph_x.copy_(x)
        self._graph_labels.copy_(labels)
        self._graph.replay()
        self.step_no += 1
        return self._graph_loss

    def _counted_step(self, lr):
        # the step argument is 0: the kernels add the device counter, which the last kernel of the step advances
        logits = self.forward(self._graph_x, 0)
        loss, dlogits = self.ops.softmax_xent(logits, self._graph_labels, 1.0 / self._graph_x.shape[0])
        self.backward(dlogits, 0, lr)
        self.ops.step_advance(self._graph_counter)
        return loss

    def calibrate(self, x, labels, adc_quantile=None):
        """Fixes x_scale / g_scale of every crossbar layer from one batch: a forward / backward pass in
        which every layer takes the maximum it sees as its range and nothing is written; the ranges
        then become those maxima times a head-room factor.  With adc_quantile a second such pass
        measures the column currents of every layer and sets the converter ranges from them."""
        self.calibrating = True
        try:
            logits = self.forward(x, 0)
            _, dlogits = self.ops.softmax_xent(logits, labels, 1.0 / x.shape[0])
            self.backward(dlogits, 0, 0.0)
        finally:
            self.calibrating = False
        for layer in self.layers:
            layer.x_scale = HEADROOM_X * layer.seen_x
            if layer.seen_g is not None:
                layer.g_scale = HEADROOM_G * layer.seen_g
        if adc_quantile is not None:
            self._measure_adc_ranges(x, labels, adc_quantile)

    def _measure_adc_ranges(self, x, labels, quantile):
        self.adc_quantile = quantile                    # the layers keep their calibrated input ranges in this pass
        self.calibrating = True                         # ... and nothing is written
        try:
            logits = self.forward(x, 0)
            _, dlogits = self.ops.softmax_xent(logits, labels, 1.0 / x.shape[0])
            self.backward(dlogits, 0, 0.0)
        finally:
            self.calibrating = False
            self.adc_quantile = None


class ResNetCifar(Network):
    def __init__(self, cfg_kwargs, batch, n_blocks=3, image=32, classes=10, widths=(16, 32, 64), seed=0, device="cuda"):
        gen = torch.Generator(device=device)
        gen.manual_seed(seed)
        self.batch, self.image, self.classes = batch, image, classes
        conv = lambda hw, cin, cout, stride, signed: CrossbarLayer(
            self, cfg_kwargs, 9 * cin, cout, xb.conv_geom(batch, hw, hw, cin, 3, 3, stride, 1), signed, gen, device)
        self.stem, self.stem_bn = conv(image, 3, widths[0], 1, True), BatchNorm(self, widths[0], device)
        self.blocks = []
        cin, hw = widths[0], image
        for stage, width in enumerate(widths):
            for b in range(n_blocks):
                stride = 2 if (b == 0 and stage > 0) else 1
                hw_out = (hw + stride - 1) // stride
                self.blocks.append(dict(a=conv(hw, cin, width, stride, False), bn_a=BatchNorm(self, width, device),
                                        b=conv(hw_out, width, width, 1, False), bn_b=BatchNorm(self, width, device),
                                        stride=stride, cin=cin, width=width))
                cin, hw = width, hw_out
        self.fc = CrossbarLayer(self, cfg_kwargs, cin, classes, None, False, gen, device)
        self.layers = [self.stem] + [blk[k] for blk in self.blocks for k in ("a", "b")] + [self.fc]
        nbytes = max(max(L.workspace_bytes(batch) for L in self.layers),
                     xb.lib().xbar_bn_workspace_bytes(batch * image * image, max(widths)), 4096)
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.step_no = 0

    # ---- forward / backward ---------------------------------------------------------------------
    def forward(self, images, step):
        ws, ops = self.ws, self.ops
        a = ops.relu_fwd(self.stem_bn.forward(self.stem.forward(images, step, ws), ws))
        self.stem_out = a
        for blk in self.blocks:
            blk["in"] = a
            h = ops.relu_fwd(blk["bn_a"].forward(blk["a"].forward(a, step, ws), ws))
            blk["mid"] = h
            h = blk["bn_b"].forward(blk["b"].forward(h, step, ws), ws)
            skip = a if (blk["stride"] == 1 and blk["cin"] == blk["width"]) else ops.shortcut_fwd(a, blk["stride"], blk["width"])
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
            h = blk["b"].backward(blk["bn_b"].backward(d, lr, ws), step, lr, ws)
            h = blk["a"].backward(blk["bn_a"].backward(ops.relu_bwd(blk["mid"], h), lr, ws), step, lr, ws)
            if blk["stride"] == 1 and blk["cin"] == blk["width"]:
                d = ops.add(h, d)
            else:
                d = ops.add(h, ops.shortcut_bwd(d, tuple(blk["in"].shape), blk["stride"]))
        d = self.stem_bn.backward(ops.relu_bwd(self.stem_out, d), lr, ws)
        self.stem.backward(d, step, lr, ws, need_dx=False)
