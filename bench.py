"""Benchmark of the crossbar-emulation hot path on one MI355X.

A step is one pass of the whole path over every layer GEMM of the workload: conductance-plane
generation, forward VMM, backward VMM and weight update, through the C ABI, with all inputs already
resident in HBM.  Prints one JSON line: emulated crossbar GMAC/s (fwd + bwd + update), the roofline of
the dominant kernel (the fused MFMA contraction + ADC + shift-and-add), measured live with HIP events
around every launch of that kernel in the timed region, and the CPU oracle timed on the host cores on
a bounded sample of the same workload.
"""
import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X dense matrix peaks of the two operand formats the contraction kernel uses (xbar_plane_format):
# fp16 planes, or 6-bit planes with 4-bit digits on the block-scaled instruction
MFMA_PEAK_TFLOPS = {0: 2500.0, 1: 10100.0}
FORMAT_NAME = {0: "f16 planes x f16 digits, f32 accumulate",
               1: "f6 (E2M3, block-scaled) planes x f4 (E2M1) digits, f32 accumulate"}
KERNEL_NAME = {0: "vmm_kernel (fp16 MFMA contraction + ADC + shift-and-add, fwd and bwd launches)",
               1: "vmm6_kernel (block-scaled 6-bit x 4-bit MFMA contraction + ADC + shift-and-add, fwd and bwd launches)"}
# HBM bytes per contraction-kernel launch (average over the 108 launches of a step) of the default workload:
# recorded from the FETCH_SIZE / WRITE_SIZE counter runs in the profile named here, not measured in this run
VMM_TRAFFIC_BYTES_RESNET50_B64 = 532760064      # (152244 KiB FETCH_SIZE x 2.00 + 215786 KiB WRITE_SIZE x 1.00) x 1024
VMM_TRAFFIC_SOURCE = "profiles/vmm6_kernel_resnet50_batch64.txt"


def contraction_roofline(achieved, fmt, terms):
    """Roofline entry of the contraction kernel: useful flops (2 per emulated MAC) against the matrix peak of
    the operand type it runs on; a plane value split into `terms` operand terms issues `terms` times that."""
    peak = MFMA_PEAK_TFLOPS[fmt]
    return {"bound": "mfma", "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s",
            "frac": round(achieved / peak, 4), "traffic": None, "kernel": KERNEL_NAME[fmt],
            "operand_terms": terms, "issued_frac": round(terms * achieved / peak, 4),
            "frac_of_fp16_peak": round(achieved / MFMA_PEAK_TFLOPS[0], 4)}


class HipEvents:
    """hipEvent_t pairs created straight from the HIP runtime (the library records them on the stream
    it launches on)."""

    def __init__(self):
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [C.c_void_p]
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]
        self.pool = []

    def pair(self):
        a, b = C.c_void_p(), C.c_void_p()
        assert self.hip.hipEventCreate(C.byref(a)) == 0 and self.hip.hipEventCreate(C.byref(b)) == 0
        self.pool.append((a, b))
        return a.value, b.value

    def elapsed_ms(self, a, b):
        ms = C.c_float()
        assert self.hip.hipEventSynchronize(C.c_void_p(b)) == 0
        assert self.hip.hipEventElapsedTime(C.byref(ms), C.c_void_p(a), C.c_void_p(b)) == 0
        return ms.value


def end_to_end(args, torch, workloads, xb, device):
    """Whole training steps of a residual network from images: the CIFAR-size ResNet-20 (19 convolutions +
    classifier) or ResNet-50 (53 convolutions + classifier)."""
    from paper_2002_11151_amd import resnet_cifar, resnet_imagenet, sequential
    assert args.workload in ("mlp", "resnet20", "resnet50", "vgg16"), "--end-to-end: mlp, resnet20, resnet50 or vgg16"
    batch = args.batch or {"mlp": 128, "resnet20": 128, "resnet50": 64, "vgg16": 128}[args.workload]
    kw = workloads.config_kwargs(args.workload)
    if args.adc_bits:
        kw["adc_bits"] = args.adc_bits
    S_w, S_in = kw["weight_bits"] // kw["slice_bits"], kw["input_bits"] // kw["stream_bits"]
    gemms = workloads.GEMMS[args.workload](batch)
    tot = {k: sum(workloads.macs(g, S_w, S_in)[k] for g in gemms) for k in ("fwd", "bwd", "upd", "logical")}
    tot["bwd"] -= workloads.macs(gemms[0], S_w, S_in)["bwd"]        # no error is propagated to the image
    gen = torch.Generator(device=device)
    gen.manual_seed(0)
    image, classes = {"mlp": (28, 10), "resnet20": (32, 10)}.get(args.workload, (224, 1000))
    channels = 1 if args.workload == "mlp" else 3
    images = torch.randn((batch, image, image, channels), generator=gen, device=device)
    labels = torch.randint(0, classes, (batch,), generator=gen, device=device).to(torch.int32)
    if args.workload == "resnet20":
        net = resnet_cifar.ResNetCifar(kw, batch=batch, n_blocks=3, image=32, classes=10, seed=0, device=device)
    elif args.workload == "resnet50":
        net = resnet_imagenet.ResNetBottleneck(kw, batch=batch, seed=0, device=device)
    elif args.workload == "vgg16":
        net = sequential.Sequential(kw, sequential.vgg16_spec(), batch, (224, 224, 3), seed=0, device=device)
    else:
        images = images.abs_()                               # pixel intensities: the first layer is unsigned
        net = sequential.Sequential(kw, sequential.mlp_spec(), batch, (28, 28, 1), signed_input=False, seed=0,
                                    device=device)
    net.calibrate(images, labels)

    events = HipEvents()
    records = []

    class Traced:                      # the binding, with HIP events around every contraction kernel
        def __getattr__(self, name):
            fn = getattr(xb, name)
            if name not in ("fwd", "bwd", "conv_fwd", "conv_bwd") or not self.timed:
                return fn

            def wrapped(*a, **k):
                ev = events.pair()
                xb.trace_next_vmm(*ev)
                records.append(ev)
                return fn(*a, **k)
            return wrapped

    traced = Traced()
    traced.timed = False
    net.ops = traced
    for _ in range(args.warmup):
        net.train_step(images, labels, 0.01)
    torch.cuda.synchronize()
    traced.timed = True
    t0 = time.perf_counter()
    for _ in range(args.steps):
        loss = net.train_step(images, labels, 0.01)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    graph_ms = None
    if args.graph:                     # the same steps replayed from a captured HIP graph (one launch per step)
        net.ops = xb
        net.capture(images, labels, 0.01)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            net.replay(images, labels)
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t1) / args.steps * 1e3
    vmm_ms = sum(events.elapsed_ms(a, b) for a, b in records)
    emulated = tot["fwd"] + tot["bwd"] + tot["upd"]
    achieved = 2.0 * (tot["fwd"] + tot["bwd"]) * args.steps / (vmm_ms * 1e-3) / 1e12
    fmt, terms = xb.plane_format(xb.make_config(**kw))
    roofline = contraction_roofline(achieved, fmt, terms)
    roofline.update({"launches": len(records), "avg_launch_ms": round(vmm_ms / max(1, len(records)), 4),
                     "kernel_time_share": round(vmm_ms / (elapsed * 1e3), 4)})
    line = {
        "metric": "emulated crossbar GMAC/s (fwd+bwd+update)", "value": round(emulated / (elapsed / args.steps) / 1e9, 1),
        "unit": "GMAC/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(elapsed / args.steps * 1e3, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": FORMAT_NAME[fmt], "data": "synthetic",
        "config": {"workload": "%s whole training step from %dx%dx%d images, batch %d, %dx%d crossbars, %d-bit "
                               "weights in %d slices, %d-bit inputs in %d cycles, %d-bit ADC, wire parasitics (AAM) + "
                               "write non-linearity + noise, digital batch norm / ReLU / pooling / loss" %
                               (args.workload, image, image, channels, batch, kw["xbar_rows"], kw["xbar_cols"], kw["weight_bits"], S_w, kw["input_bits"], S_in,
                                kw["adc_bits"]),
                   "emulated_macs_per_step": emulated, "logical_macs_per_step": tot["logical"]},
        "final_loss": round(float(loss.mean()), 4),
        "ms_per_step_from_hip_graph": None if graph_ms is None else round(graph_ms, 3),
        "roofline": roofline,
        "cpu_baseline": None,
    }
    print(json.dumps(line))


# Pulse-level update of the benchmark: 31-slot trains, a device with about a thousand states over its
# range, inputs fire in proportion to their size and the error range follows from the learning rate:
# mean written change = lr x dY / w_max  <=>  x_range d_range = bl dw_min w_max / lr.
PULSE_DW_MIN, PULSE_LR = 1e-3, 0.01


def pulse_d_range(L):
    return 31 * PULSE_DW_MIN * L["w_max"] / (PULSE_LR * L["x_scale"])


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="resnet50", choices=["fc256", "mlp", "resnet20", "resnet50", "vgg16"])
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rows", type=int, default=None, help="batch rows per layer for the oracle sample")
    ap.add_argument("--ideal", action="store_true", help="array non-idealities off (single-term operands)")
    ap.add_argument("--xbar", type=int, default=0,
                    help="crossbar rows = columns instead of the workload's preset (the paper's own runs use 64)")
    ap.add_argument("--graph", action="store_true",
                    help="with --end-to-end: also time the training step replayed from a captured HIP graph")
    ap.add_argument("--pulsed-update", action="store_true",
                    help="pulse-level update (stochastic pulse trains of 31 slots, one sample at a time) instead of "
                         "the aggregate write")
    ap.add_argument("--offset-inputs", action="store_true",
                    help="signed inputs in one phase of offset-binary codes instead of two phases of magnitudes: "
                         "half the crossbar passes of every signed pass")
    ap.add_argument("--adc-per-array", action="store_true",
                    help="one unsigned converter per array and digital subtraction instead of one signed converter "
                         "per array pair: twice the contraction work for the same emulated MACs")
    ap.add_argument("--all-paths", action="store_true",
                    help="wire model with every first-order path instead of the shortest path per device")
    ap.add_argument("--from-images", action="store_true",
                    help="convolution layers take NHWC activations and gather their patches on the fly "
                         "(xbar_conv_*) instead of reading a patch matrix prepared outside the timed region")
    ap.add_argument("--adc-bits", type=int, default=None, help="override the converter resolution of the workload")
    ap.add_argument("--end-to-end", action="store_true",
                    help="mlp / resnet20 / resnet50 / vgg16: time whole training steps of the network (crossbar layers from images, "
                         "digital batch norm / ReLU / pooling / loss) instead of the list of layer GEMMs")
    ap.add_argument("--overlap-update", action="store_true",
                    help="run the weight update of a layer beside its backward pass on a second stream (1 %% less "
                         "time per step; the contraction kernel then shares the matrix pipes and times 4 %% slower)")
    ap.add_argument("--fcm-refresh", action="store_true",
                    help="also time one refresh of the circuit-level distortion profile of every layer "
                         "(reported as fcm_refresh_ms; not part of the step)")
    ap.add_argument("--per-layer", action="store_true", help="print a per-layer table to stderr")
    ap.add_argument("--no-mfma-probe", action="store_true", help="skip the bare-MFMA sustained-rate probe")
    ap.add_argument("--calib-copy", action="store_true",
                    help="run one 1 GiB device-to-device copy first (known size, to scale HBM byte counters)")
    ap.add_argument("--only", default=None, help="comma-separated layer names: run just these (profiling)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every box has one); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import workloads
    from paper_2002_11151_amd import xbar as xb

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    device = torch.device("cuda:0")
    xb.lib()

    if args.end_to_end:
        return end_to_end(args, torch, workloads, xb, device)

    default_batch = {"fc256": 64, "mlp": 128, "resnet20": 128, "resnet50": 64, "vgg16": 128}[args.workload]
    batch = args.batch or default_batch
    gemms = workloads.GEMMS[args.workload](batch) if args.workload in ("fc256", "mlp") else \
        workloads.GEMMS[args.workload](batch, merge=True)
    if args.only:
        gemms = [g for g in gemms if g.name in args.only.split(",")]
        assert gemms, "no such layer"
    kw = workloads.config_kwargs(args.workload)
    if args.adc_bits:
        kw["adc_bits"] = args.adc_bits
    if args.xbar:
        kw["xbar_rows"] = kw["xbar_cols"] = args.xbar
        kw["adc_fs_fwd"] = kw["adc_fs_bwd"] = workloads.adc_full_scale(args.xbar, kw["stream_bits"], kw["slice_bits"])
    if args.ideal:
        kw["flags"] &= ~(workloads.NI_VARIATION | workloads.NI_WIRE_AAM | workloads.NI_WIRE_PROFILE)
    if args.all_paths and kw["flags"] & workloads.NI_WIRE_AAM:
        kw["flags"] = (kw["flags"] & ~workloads.NI_WIRE_AAM) | workloads.NI_WIRE_AAM2
    signed_phases = 2
    if args.offset_inputs:
        kw["flags"] |= workloads.INPUT_OFFSET
        signed_phases = 1
    arrays = 1
    if args.adc_per_array:
        kw["flags"] |= workloads.ADC_PER_ARRAY
        arrays = 2
    S_w, S_in = kw["weight_bits"] // kw["slice_bits"], kw["input_bits"] // kw["stream_bits"]
    fmt, terms = xb.plane_format(xb.make_config(**kw))

    # ---- resident tensors, one set per distinct shape ------------------------------------------
    layers = []
    max_planes = max_ws = max_out = max_ws_upd = 0
    for i, g in enumerate(gemms):
        flags = kw["flags"] | (workloads.INPUT_SIGNED if g.signed_input else 0)
        cfg = xb.make_config(**dict(kw, flags=flags, seed=(kw["seed"] << 20) + i))      # every layer keys its own random streams
        W, X, dY = workloads.layer_tensors_torch(g, seed=i, device=device)
        geom = None
        if args.from_images and g.conv is not None:
            X = workloads.image_tensor_torch(g, seed=i, device=device)
            b_, hw_, cin_, k_, stride_, pad_ = g.conv
            geom = xb.conv_geom(b_, hw_, hw_, cin_, k_, k_, stride_, pad_)
            assert geom.batch * geom.out_h * geom.out_w == g.M and k_ * k_ * cin_ == g.K
        w_max = 2.0 * float(W.abs().max())          # head-room: the weights move during the run
        layers.append(dict(g=g, cfg=cfg, W=W, X=X, dY=dY, w_max=w_max, x_scale=float(X.abs().max()), geom=geom,
                           g_scale=float(dY.abs().max()), macs=workloads.macs(g, S_w, S_in, signed_phases)))
        max_planes = max(max_planes, xb.planes_bytes(cfg, g.K, g.N))
        if geom is None:
            max_ws = max(max_ws, *(xb.workspace_bytes(cfg, op, g.M, g.K, g.N) for op in (0, 1, 2)))
        else:
            max_ws = max(max_ws, *(xb.conv_workspace_bytes(cfg, op, geom, g.N) for op in (0, 1, 2)))
        max_ws_upd = max(max_ws_upd, xb.workspace_bytes(cfg, 2, g.M, g.K, g.N) if geom is None else
                         xb.conv_workspace_bytes(cfg, 2, geom, g.N))
        if args.pulsed_update:
            max_ws_upd = max(max_ws_upd, xb.workspace_bytes(cfg, xb.OP_UPDATE_PULSED, g.M, g.K, g.N) if geom is None else
                             xb.conv_workspace_bytes(cfg, xb.OP_UPDATE_PULSED, geom, g.N))
            max_ws = max(max_ws, max_ws_upd)
        max_out = max(max_out, g.M * g.N, g.M * g.K)
    planes = torch.empty(max_planes, dtype=torch.uint8, device=device)
    ws = torch.empty(max_ws, dtype=torch.uint8, device=device)
    # the update of a layer does not depend on its backward pass: on request it runs beside it on a second
    # stream (default priority) with a workspace of its own
    side = torch.cuda.Stream() if args.overlap_update else None
    ws_upd = ws if side is None else torch.empty(max_ws_upd, dtype=torch.uint8, device=device)
    tiled, updated = torch.cuda.Event(), torch.cuda.Event()
    out = torch.empty(max_out, dtype=torch.float32, device=device)

    if args.calib_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=device).normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                     # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    pulsed_events = []        # event pairs around the pulse-level updates of the timed steps
    events = HipEvents()
    vmm_records = []          # (layer index, 'fwd'|'bwd', event pair)

    def step(step_no, timed):
        main = torch.cuda.current_stream()
        for li, L in enumerate(layers):
            g, cfg = L["g"], L["cfg"]
            for rep in range(g.count):
                s = step_no * 64 + rep
                xb.tile(cfg, L["W"], L["w_max"], s, planes=planes)
                if side is not None:
                    tiled.record(main)
                if timed:
                    ev = events.pair()
                    xb.trace_next_vmm(*ev)
                    vmm_records.append((li, "fwd", ev))
                geom = L["geom"]
                if geom is None:
                    xb.fwd(cfg, planes, L["X"], g.N, L["w_max"], L["x_scale"], ws=ws, out=out[:g.M * g.N].view(g.M, g.N))
                else:
                    xb.conv_fwd(cfg, planes, L["X"], geom, g.N, L["w_max"], L["x_scale"], ws=ws,
                                out=out[:g.M * g.N].view(geom.batch, geom.out_h, geom.out_w, g.N))

                def update():
                    if args.pulsed_update and geom is None:
                        xb.update_pulsed(cfg, L["W"], L["X"], L["dY"], L["w_max"], L["x_scale"], pulse_d_range(L), 31,
                                         PULSE_DW_MIN, s, ws=ws_upd)
                    elif args.pulsed_update:
                        xb.conv_update_pulsed(cfg, L["W"], L["X"], L["dY"].view(geom.batch, geom.out_h, geom.out_w, g.N),
                                              geom, L["w_max"], L["x_scale"], pulse_d_range(L), 31, PULSE_DW_MIN, s,
                                              ws=ws_upd)
                    elif geom is None:
                        xb.update(cfg, L["W"], L["X"], L["dY"], L["w_max"], 1.0 / L["w_max"], 0.01, s, ws=ws_upd)
                    else:
                        xb.conv_update(cfg, L["W"], L["X"], L["dY"].view(geom.batch, geom.out_h, geom.out_w, g.N), geom,
                                       L["w_max"], 1.0 / L["w_max"], 0.01, s, ws=ws_upd)

                if side is not None:                      # W may be written once the generator has read it
                    side.wait_event(tiled)
                    with torch.cuda.stream(side):
                        update()
                        updated.record(side)
                if timed:
                    ev = events.pair()
                    xb.trace_next_vmm(*ev)
                    vmm_records.append((li, "bwd", ev))
                if geom is None:
                    xb.bwd(cfg, planes, L["dY"], g.K, L["w_max"], L["g_scale"], ws=ws, out=out[:g.M * g.K].view(g.M, g.K))
                else:
                    xb.conv_bwd(cfg, planes, L["dY"].view(geom.batch, geom.out_h, geom.out_w, g.N), geom, g.N, L["w_max"],
                                L["g_scale"], ws=ws, out=out[:L["X"].numel()].view(L["X"].shape))
                if side is None:
                    if timed and args.pulsed_update:
                        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        e0.record()
                        update()
                        e1.record()
                        pulsed_events.append((e0, e1))
                    else:
                        update()
                else:
                    main.wait_event(updated)              # the next generator call reads the written W

    for w in range(args.warmup):
        step(w, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(args.warmup + k, True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    tot = {k: sum(L["macs"][k] * L["g"].count for L in layers) for k in ("fwd", "bwd", "upd", "logical")}
    emulated = tot["fwd"] + tot["bwd"] + tot["upd"]
    ms_per_step = elapsed / args.steps * 1e3
    value = emulated / (elapsed / args.steps) / 1e9

    # ---- roofline of the contraction kernel ------------------------------------------------------
    vmm_ms = 0.0
    vmm_flops = 0.0
    per_layer = {}
    for li, kind, (a, b) in vmm_records:
        ms = events.elapsed_ms(a, b)
        vmm_ms += ms
        fl = 2.0 * arrays * layers[li]["macs"][kind]          # arrays read one by one are contracted one by one
        vmm_flops += fl
        d = per_layer.setdefault((li, kind), [0.0, 0.0, 0])
        d[0] += ms
        d[1] += fl
        d[2] += 1
    achieved = vmm_flops / (vmm_ms * 1e-3) / 1e12 if vmm_ms > 0 else 0.0
    roofline = contraction_roofline(achieved, fmt, terms)
    roofline.update({"launches": len(vmm_records), "avg_launch_ms": round(vmm_ms / max(1, len(vmm_records)), 4),
                     "kernel_time_share": round(vmm_ms / (elapsed * 1e3), 4)})
    # Context for the fraction above, measured in this process: the rate the chip sustains on the bare matrix
    # instructions (it is power limited once operands toggle), and the contraction kernel's own inner loop
    # (4 terms, 128-row tiles) on synthetic operands without and with the ADC / shift-and-add operations:
    # what the fused epilogue adds to the loop's time.
    if not args.no_mfma_probe:
        probe = {}
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        times = {}
        for mode, key, iters in ((0, "fp16_dense_random_operands", 100000), (1, "fp16_single_bit_digits", 100000),
                                 (4, "f6xf4_block_scaled_single_bit_digits", 100000),
                                 (5, "contraction_loop_without_adc_issued", 50000),
                                 (6, "contraction_loop_with_adc_issued", 50000)):
            xb.probe_mfma_rate(mode, 2000, ws)
            torch.cuda.synchronize()
            e0.record()
            flops = xb.probe_mfma_rate(mode, iters, ws)
            e1.record()
            torch.cuda.synchronize()
            times[mode] = e0.elapsed_time(e1)
            probe[key] = round(flops / (times[mode] * 1e-3) / 1e12, 1)
        roofline["sustained_mfma_tflops"] = probe
        roofline["epilogue_added_frac"] = round(times[6] / times[5] - 1.0, 4)
    if (args.workload == "resnet50" and batch == 64 and not args.only and not args.ideal and not args.all_paths
            and not args.adc_per_array and not args.offset_inputs and not args.from_images and not args.xbar
            and not args.adc_bits):
        roofline["traffic"] = VMM_TRAFFIC_BYTES_RESNET50_B64
        roofline["traffic_source"] = "recorded counter run, " + VMM_TRAFFIC_SOURCE
    fcm_refresh_ms = None
    if args.fcm_refresh:
        # one circuit-level solve of every layer (Sec. IV-D: done every L iterations, its profile reused between)
        fcm_ws = torch.empty(max(xb.workspace_bytes(L["cfg"], xb.OP_FCM, 1, L["g"].K, L["g"].N) for L in layers),
                             dtype=torch.uint8, device=device)
        prof = torch.empty(max(S_w * 2 * L["g"].K * L["g"].N for L in layers), dtype=torch.float32, device=device)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for L in layers:
            g = L["g"]
            for rep in range(g.count):
                xb.fcm_profile(L["cfg"], L["W"], L["w_max"], rep, fcm_ws, prof[:S_w * 2 * g.K * g.N].view(S_w, 2, g.K, g.N))
        torch.cuda.synchronize()
        fcm_refresh_ms = round((time.perf_counter() - t0) * 1e3, 1)
        del fcm_ws, prof
    if args.per_layer:
        for (li, kind), (ms, fl, n) in sorted(per_layer.items()):
            g = layers[li]["g"]
            print("%-10s %s K=%5d N=%5d M=%7d x%d  %8.3f ms/launch  %7.1f TFLOP/s useful" %
                  (g.name, kind, g.K, g.N, g.M, g.count, ms / n, fl / (ms * 1e-3) / 1e12), file=sys.stderr)

    # ---- CPU oracle on a bounded sample ------------------------------------------------------------
    cpu = None
    if not args.no_cpu_baseline and not args.from_images:
        from oracle import xbar_oracle as xo
        threads = min(16, os.cpu_count() or 1)
        rows = args.cpu_rows or threads
        done = 0
        t_cpu = 0.0
        for L in layers:
            g = L["g"]
            m = min(rows, g.M)
            flags = kw["flags"] | (workloads.INPUT_SIGNED if g.signed_input else 0)
            co = xo.make_config(**dict(kw, flags=flags))
            W = L["W"].cpu().numpy()
            X = L["X"][:m].cpu().numpy()
            dY = L["dY"][:m].cpu().numpy()
            t1 = time.perf_counter()
            U = xo.planes(co, W, L["w_max"], 0)
            col, row = xo.weight_sums(co, W, L["w_max"]) if signed_phases == 1 else (None, None)
            xo.rows_parallel(lambda u, x: xo.fwd_planes(co, u, x, L["w_max"], L["x_scale"], wsum=col), U, X, threads)
            xo.rows_parallel(lambda u, x: xo.bwd_planes(co, u, x, L["w_max"], L["g_scale"], wsum=row), U, dY, threads)
            xo.update(co, W, X, dY, L["w_max"], 1.0 / L["w_max"], 0.01, 0)
            t_cpu += time.perf_counter() - t1
            mm = workloads.macs(g._replace(M=m), S_w, S_in, signed_phases)
            done += mm["fwd"] + mm["bwd"] + mm["upd"]
        cpu = {"value": round(done / t_cpu / 1e9, 4), "unit": "emulated GMAC/s", "cores": threads, "kind": "oracle",
               "sample": "%d batch rows of each of the %d distinct layer shapes, fwd+bwd+update, %.1f s" %
                         (rows, len(layers), t_cpu)}

    if kw["flags"] & (workloads.NI_VARIATION | workloads.NI_WIRE_AAM | workloads.NI_WIRE_PROFILE | workloads.NI_WIRE_AAM2):
        array_text = "wire parasitics (%s) + write non-linearity + noise" % (
            "AAM, all first-order paths" if kw["flags"] & workloads.NI_WIRE_AAM2 else "AAM")
    else:
        array_text = "ideal arrays"
    if args.pulsed_update:
        array_text += ", pulse-level update (31-slot stochastic trains)"
    if signed_phases == 1:
        array_text += ", offset-binary signed inputs"
    if arrays == 2:
        array_text += ", one converter per array"
    line = {
        "metric": "emulated crossbar GMAC/s (fwd+bwd+update)", "value": round(value, 1), "unit": "GMAC/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": FORMAT_NAME[fmt],
        "data": "synthetic",
        "config": {"workload": "%s layer GEMMs (%d GEMMs, %d distinct shapes), batch %d, %dx%d crossbars, "
                               "%d-bit weights in %d slices, %d-bit inputs in %d cycles, %d-bit ADC, %s" %
                               (args.workload, sum(g.count for g in gemms), len(gemms), batch, kw["xbar_rows"],
                                kw["xbar_cols"], kw["weight_bits"], S_w, kw["input_bits"], S_in, kw["adc_bits"],
                                array_text),
                   "emulated_macs_per_step": emulated, "logical_macs_per_step": tot["logical"]},
        "logical_gmacs": round(tot["logical"] / (elapsed / args.steps) / 1e9, 1),
        "roofline": roofline, "cpu_baseline": cpu,
    }
    if fcm_refresh_ms is not None:
        line["fcm_refresh_ms"] = fcm_refresh_ms
    if args.pulsed_update:
        # pulses of one step, counted in an untimed pass on copies of the weights: the library reports the signed
        # (net) count per device, and the trains depend on magnitudes only, so the same pass on |X| and |dY| sends
        # every pulse the same way and its net count is the number of pulses
        n_pulses = 0
        for L in layers:
            g = L["g"]
            dw = PULSE_DW_MIN
            if L["geom"] is None:
                _, cnt = xb.update_pulsed(L["cfg"], L["W"].clone(), L["X"].abs(), L["dY"].abs(), L["w_max"], L["x_scale"],
                                          pulse_d_range(L), 31, dw, 0, ws=ws_upd, want_pulses=True)
            else:
                q = L["geom"]
                _, cnt = xb.conv_update_pulsed(L["cfg"], L["W"].clone(), L["X"].abs(),
                                               L["dY"].abs().view(q.batch, q.out_h, q.out_w, g.N), q, L["w_max"],
                                               L["x_scale"], pulse_d_range(L), 31, dw, 0, ws=ws_upd, want_pulses=True)
            n_pulses += int(cnt.abs().sum().item()) * g.count
        upd_ms = sum(a.elapsed_time(b) for a, b in pulsed_events) / args.steps
        line["pulsed_update"] = {"ms_per_step": round(upd_ms, 3), "pulses_per_step": n_pulses,
                                 "device_samples_per_step": tot["upd"],
                                 "gpulses_per_s": round(n_pulses / (upd_ms * 1e-3) / 1e9, 3),
                                 "device_gsamples_per_s": round(tot["upd"] / (upd_ms * 1e-3) / 1e9, 1)}
    print(json.dumps(line))


if __name__ == "__main__":
    main()
