#!/usr/bin/env python3
"""Throughput of the TSM-ResNet-50 train step (forward + backward + SGD update) on one MI355X.

One "step" = one call of tsm_resnet50_step on a batch of synthetic Kinetics-shaped clips
(8 frames of 3x224x224, 400 classes) that is already resident in HBM.  Prints ONE JSON line with the
throughput in clips/s, a roofline object for the kernel class that takes the most time (its time
measured live with HIP events on the launch stream), and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, published
STAGES = (("res2", 3, 64, 1), ("res3", 4, 128, 2), ("res4", 6, 256, 2), ("res5", 3, 512, 2))


def conv_layers(F, size):
    """(name, rows_in, Cin, rows_out, Cout, taps, has_dgrad) of the 53 convolutions for F frames."""
    h = size // 2
    layers = [("conv1", F * size * size, 3, F * h * h, 64, 49, False)]
    h //= 2
    cin = 64
    for name, blocks, mid, stride in STAGES:
        for b in range(blocks):
            s = stride if b == 0 else 1
            ho = h // s
            pre = "%s.%d." % (name, b)
            layers.append((pre + "c1", F * h * h, cin, F * h * h, mid, 1, True))
            layers.append((pre + "c2", F * h * h, mid, F * ho * ho, mid, 9, True))
            layers.append((pre + "c3", F * ho * ho, mid, F * ho * ho, 4 * mid, 1, True))
            if b == 0:
                layers.append((pre + "ds", F * h * h, cin, F * ho * ho, 4 * mid, 1, True))
            cin, h = 4 * mid, ho
    return layers


def pw_layer(cs, cd, rows):
    """Shapes the short-K, wide-result 1x1 kernels take: K of 64, 128 or 256 channels, a result at least twice as wide
    (a block holds 256 of its channels, 128 at K = 256), a pass of 32 pixels for every wavefront of the grid."""
    if cs not in (64, 128, 256) or not 256 <= cd <= 1024 or cd < 2 * cs:
        return False
    nb = 256 if cs <= 128 else 128
    return cd % nb == 0 and rows >= 32 * 8 * 256 // (cd // nb)


def igemm_class(kind, cd, cs, rows, taps=1, stride=1, affine=False):
    """Kernel and tile the library picks for a forward ("fwd") or data-gradient ("dgrad") convolution that produces
    `rows` pixels of `cd` channels from `cs` source channels (tensors below 2 GiB, which holds for every workload
    here; 256 CUs).  affine: a forward layer with the affine epilogue of the inference path, which the 256-column tiles
    and the short-K kernel at K = 128 do not carry."""
    if stride == "stem":      # the space-to-depth stem: its own kernel from five rounds of tiles on
        return "igemm_fwd_stem" if -(-rows // 256) >= 5 * 256 else "igemm_fwd_256x64"
    if cs % 64 == 0:
        tiles256 = -(-rows // 256) * (1 if cd <= 64 else -(-cd // 128))
        r = "r128" if tiles256 * 4 < 256 * 3 else "256"
        if cs == 64 and cd == 64 and taps == 9 and stride == 1 and -(-rows // 256) >= 5 * 256:
            return "igemm_%s_c64" % kind      # the 64 -> 64 channel 3x3 kernel (five rounds of tiles or more)
        if kind == "fwd" and not (affine and cs == 128) and taps == 1 and stride == 1 and r == "256" and pw_layer(cs, cd, rows):
            return "igemm_fwd_pw"             # the short-K 1x1 forward kernel (affine epilogue: K = 64 and 256 only)
        if kind == "fwd" and not affine and cd % 256 == 0 and r == "256" and -(-rows // 256) * (cd // 256) * 2 >= 256:
            return "igemm_fwd_256x256"        # wide results: 256-column tiles from half a round on
        # 64 columns per tile for narrow outputs, and where even 128x128 tiles leave a quarter of the CUs idle
        narrow = cd <= 64 or (r == "r128" and -(-rows // 128) * -(-cd // 128) * 4 < 256 * 3)
        return "igemm_%s_%sx%s" % (kind, r, "64" if narrow else "128")
    return "igemm_%s_%s" % (kind, "128x64" if cd <= 64 else "128x128")


def wgrad_class(cout, cin, taps):
    """Tile the library picks for a weight gradient (`cin` as stored: the stem's 3 channels are padded to 8)."""
    kk = taps * cin
    if cin % 64 == 0 and cout % 64 == 0:
        if cout % 256 == 0:
            return "wgrad_tr_256x128" if cin % 128 == 0 else "wgrad_tr_256x64"
        if cout % 128 == 0 and cin % 128 == 0:
            return "wgrad_tr_128x128"
        if cin % 256 == 0:
            return "wgrad_tr_64x256"
        if taps == 1:
            return "wgrad_tr_64x64"
        if kk % 192 == 0:
            return "wgrad_tr_64x192"
    if cout > 64 and kk > 64:
        return "wgrad_128x128"
    return "wgrad_64x192" if (cout <= 64 and kk >= 192 and kk % 192 == 0) else "wgrad_64x64"


def dgrad_class(name, rin, cin, rout, cout, taps):
    """Class of a layer's data gradient.  A strided 1x1 projection sends gradient only to the input pixels with even
    row and column: the library computes it as a stride-1 data gradient on the output grid (compact form)."""
    if name.endswith(".ds") and rin != rout:
        return igemm_class("dgrad", cin, cout, rout, 1, 1)
    # the first convolution of a block, short in K and wide in its result: the kernel of its own (behind a strided
    # projection, whose gradient arrives in compact form, the variants for 128 and 256 source channels)
    if name.endswith(".c1") and taps == 1 and rin == rout and pw_layer(cout, cin, rin):
        tiles256 = -(-rin // 256) * -(-cin // 128)
        if tiles256 * 4 >= 256 * 3:
            return "igemm_dgrad_pw"
    return igemm_class("dgrad", cin, cout, rin, taps, 1 if rin == rout else 2)


def class_work(F, size):
    """Algorithmic FLOPs per step of each MFMA kernel class (2 x multiply-accumulates of the layers it
    runs) -- counted from the layer table, never from padded tiles."""
    work = {}

    def add(cls, macs):
        work[cls] = work.get(cls, 0.0) + 2.0 * macs

    for name, rin, cin, rout, cout, taps, has_dgrad in conv_layers(F, size):
        macs = float(rout) * cout * cin * taps
        stem = name == "conv1"   # runs in space-to-depth form: 64 "channels" x 4 taps, see the library
        add(igemm_class("fwd", cout, 64 if stem else cin, rout, taps, "stem" if stem else (1 if rin == rout else 2)), macs)
        if has_dgrad:
            add(dgrad_class(name, rin, cin, rout, cout, taps), macs)
        add("wgrad_tr_64x256" if stem else wgrad_class(cout, cin, taps), macs)
    return work


def class_bytes(F, size, epilogue_reads=True):
    """Algorithmic HBM bytes per step of each MFMA kernel class: every layer reads its two operands once
    and writes its result once (bf16 activations; weight-sized tensors are negligible and left out).
    epilogue_reads: also count the tensors a fused data-gradient epilogue reads."""
    byt = {}

    def add(cls, b):
        byt[cls] = byt.get(cls, 0.0) + b

    for name, rin, cin, rout, cout, taps, has_dgrad in conv_layers(F, size):
        stem = name == "conv1"
        x_b, y_b = 2.0 * rin * cin, 2.0 * rout * cout
        if stem:   # the space-to-depth image: (size/2 + 3)^2 pixels of 16 values per frame
            x_b = 2.0 * F * (size // 2 + 3) ** 2 * 16
        # (a strided 1x1 projection reads, and its gradients read or write, only the input pixels with even row and column)
        xs_b = x_b / 4.0 if (name.endswith(".ds") and rin != rout) else x_b
        add(igemm_class("fwd", cout, 64 if stem else cin, rout, taps, "stem" if stem else (1 if rin == rout else 2)), xs_b + y_b)
        if has_dgrad:
            extra = x_b if name.endswith(".c1") else 0.0       # the shortcut gradient added in the epilogue
            blk0 = int(name.split(".")[1]) == 0
            if name.endswith(".c1") and blk0 and not name.startswith("res2"):
                extra = x_b / 4.0                              # ... in compact form behind a strided projection
            dx_b = xs_b                                        # (the compact form is what is written)
            # ReLU mask and BatchNorm sums of the layer below ride in the epilogue (two more tensors of the
            # result's size are read): always for c2 / c3, for c1 when the block below has an identity shortcut
            blk = int(name.split(".")[1])
            chained = name.endswith(".c1") and (blk >= 2 or (blk == 0 and not name.startswith("res2")))
            # (a block's output mask is read as decision bits, a sixteenth of the tensor; inside a block the
            # activation itself is the mask)
            if name.endswith((".c2", ".c3")):
                extra += 2.0 * x_b
            elif chained:
                extra += x_b + x_b / 16.0
            elif name.endswith(".c1") and blk == 1:
                extra += x_b / 16.0    # the block below has a projection shortcut: only its ReLU mask rides along
            add(dgrad_class(name, rin, cin, rout, cout, taps), dx_b + y_b + (extra if epilogue_reads else 0.0))
        # (the stem's weight gradient forms its dy while loading: it reads dz and the BatchNorm input instead)
        add("wgrad_tr_64x256" if stem else wgrad_class(cout, cin, taps), xs_b + (2.0 if stem else 1.0) * y_b)
    return byt


def elementwise_bytes(F, size):
    """Algorithmic bytes per step of the stand-alone elementwise classes of the train step (bf16 tensors; y_b = one
    convolution output): what each pass has to read and write once."""
    byt = {"bn_bwd_apply": 0.0, "block_tail_fwd": 0.0, "bn_relu_apply": 0.0, "relu_bn_bwd_reduce": 0.0}
    layers = conv_layers(F, size)
    last_block = layers[-1][0].rsplit(".", 1)[0]
    for name, rin, cin, rout, cout, taps, has_dgrad in layers:
        if name == "conv1":
            continue          # the stem's BatchNorm backward is formed in its weight gradient's loader
        y_b = 2.0 * rout * cout
        blk, lay = name.rsplit(".", 1)
        proj = any(n == blk + ".ds" for n, *_ in layers)
        # BatchNorm backward map dy = a*dz + b*y + c: two tensors in, one out; a projection's map shares the read of
        # the upstream gradient with the block's last layer
        byt["bn_bwd_apply"] += 2.0 * y_b if lay == "ds" else 3.0 * y_b
        if lay in ("c1", "c2"):
            byt["bn_relu_apply"] += 2.0 * y_b                     # z = ReLU(BatchNorm(y))
        if lay == "c3":
            byt["block_tail_fwd"] += 3.0 * y_b + y_b / 16.0       # BatchNorm output + shortcut -> ReLU, decision bits
            if proj:
                byt["relu_bn_bwd_reduce"] += 3.0 * y_b            # masked gradient and the two BatchNorm inputs
            elif blk == last_block:
                byt["relu_bn_bwd_reduce"] += 4.0 * y_b            # gradient, block output, BatchNorm input in; dz out
    return byt


def measured_traffic(clips):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary (FETCH_SIZE + WRITE_SIZE, scaled by
    the copy-kernel calibration stated there); None when no summary for this workload is committed."""
    path = os.path.join(ROOT, "profiles", "tsm_resnet50_step_%dclips_hbm_traffic.txt" % clips)
    out = {}
    if os.path.exists(path):
        for line in open(path):
            parts = line.split()
            if len(parts) == 3 and parts[0] == "traffic_bytes_per_launch":
                out[parts[1]] = float(parts[2])
    return out


def block_workload(args, torch, B, I):
    """Block-level workloads through tsm_block_fwd / tsm_block_bwd (bf16, channels innermost, inputs resident)."""
    stream = torch.cuda.current_stream()

    def make(kind, N, T, Cin, H, Cmid, Cout, fd, seed):
        d = B.BlockDesc(kind=kind, N=N, T=T, Cin=Cin, H=H, W=H, Cmid=Cmid, Cout=Cout, stride=1, has_projection=0,
                        fold_div=fd, dtype=B.TSM_BF16, layout=B.TSM_NTHWC, bn_eps=1e-5)
        t3 = kind == B.TSM_BLOCK_BOTTLENECK_T3
        shapes = {"w1": (Cmid, Cin, 3) if t3 else (Cmid, Cin, 1, 1), "w2": (Cmid, Cmid, 3, 3), "w3": (Cout, Cmid, 1, 1)}
        p = {k: torch.from_numpy(I.kaiming_conv(v, seed + i, "bf16")).to(torch.bfloat16).cuda()
             for i, (k, v) in enumerate(shapes.items())}
        for i, c in (("1", Cmid), ("2", Cmid), ("3", Cout)):
            p["g" + i] = torch.ones(c, dtype=torch.float32, device="cuda")
            p["b" + i] = torch.zeros(c, dtype=torch.float32, device="cuda")
        g = {"d" + k: torch.empty(v.shape, dtype=torch.float32, device="cuda") for k, v in p.items()}
        saved = torch.empty(B.tsm_block_saved_bytes(d), dtype=torch.uint8, device="cuda")
        ws = torch.empty(B.tsm_block_workspace_bytes(d), dtype=torch.uint8, device="cuda")
        macs = float(N * T * H * H) * (Cin * Cmid * (3 if t3 else 1) + 9 * Cmid * Cmid + Cmid * Cout)
        return {"d": d, "p": p, "g": g, "saved": saved, "ws": ws, "flops": 6.0 * macs}

    def act(N, T, C, H, seed):
        return torch.from_numpy(I.normal((N, T, H, H, C), seed, "bf16")).to(torch.bfloat16).cuda()

    def time_it(fn):
        for _ in range(args.warmup):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(stream)
        for _ in range(args.steps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps

    base = {"n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic"}
    if args.workload == "res2":
        N, T, C, H = 8, 8, 256, 56
        blocks = [make(B.TSM_BLOCK_BOTTLENECK, N, T, C, H, 64, C, 8, 10 * i) for i in range(3)]
        xs = [act(N, T, C, H, 0)] + [torch.empty(N, T, H, H, C, dtype=torch.bfloat16, device="cuda") for _ in range(3)]
        gs = [act(N, T, C, H, 3)] + [torch.empty(N, T, H, H, C, dtype=torch.bfloat16, device="cuda") for _ in range(3)]

        def it():
            for i, b in enumerate(blocks):
                B.tsm_block_fwd(b["d"], xs[i], b["p"], xs[i + 1], b["saved"], b["ws"], stream)
            for i in (2, 1, 0):
                b = blocks[i]
                B.tsm_block_bwd(b["d"], xs[i], xs[i + 1], gs[2 - i], b["saved"], b["p"], gs[3 - i], b["g"], b["ws"], stream)

        ms = time_it(it)
        fl = sum(b["flops"] for b in blocks)
        out = dict(base, metric="TSM res2 bottleneck stack (3 blocks) fwd+bwd clips/s", value=N / (ms * 1e-3),
                   unit="clips/s", ms_per_step=ms,
                   config={"workload": "configs[1]: x[8,8,256,56,56] bf16, 256->64->64->256, fold_div 8, three blocks"},
                   tflops=fl / (ms * 1e-3) / 1e12, pct_bf16_mfma_peak=100.0 * fl / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS)
        return out
    N, T, C, H = 8, 8, 1024, 14
    res = {}
    for name, kind, fd in (("tsm", B.TSM_BLOCK_BOTTLENECK, 8), ("t3", B.TSM_BLOCK_BOTTLENECK_T3, 0)):
        b = make(kind, N, T, C, H, 256, C, fd, 1)
        x, dout = act(N, T, C, H, 0), act(N, T, C, H, 3)
        o, dx = torch.empty_like(x), torch.empty_like(x)

        def it():
            B.tsm_block_fwd(b["d"], x, b["p"], o, b["saved"], b["ws"], stream)
            B.tsm_block_bwd(b["d"], x, o, dout, b["saved"], b["p"], dx, b["g"], b["ws"], stream)

        ms = time_it(it)
        res[name] = {"ms": ms, "tflops": b["flops"] / (ms * 1e-3) / 1e12}
    out = dict(base, metric="TSM block fwd+bwd clips/s at x[8,8,1024,14,14] (3x1x1 temporal-conv block beside it)",
               value=N / (res["tsm"]["ms"] * 1e-3), unit="clips/s", ms_per_step=res["tsm"]["ms"],
               config={"workload": "configs[4]: bottleneck 1024->256->256->1024 at 14x14, 8 clips x 8 frames, bf16"},
               tsm_block=res["tsm"], temporal_conv_block=res["t3"],
               t3_over_tsm_time=res["t3"]["ms"] / res["tsm"]["ms"])
    return out


def infer_workload(args, torch, B, I):
    """Forward-only throughput, BatchNorm in inference mode, as the paper's efficiency table measures it
    (section 3a, Table 1: videos per second at batch 16 on one GPU)."""
    N, T, S, K = args.clips, 8, 224, 400
    table = B.tsm_resnet50_param_table(K)
    flat = I.init_params([(n, s) for n, _, s, _ in table], 1)
    d = B.R50Desc(N=N, T=T, size=S, num_classes=K, fold_div=8, lr=0.0, momentum=0.9, weight_decay=1e-4, bn_eps=1e-5,
                  bn_momentum=0.1, dtype=B.TSM_BF16)
    ws = torch.empty(B.tsm_resnet50_infer_workspace_bytes(d), dtype=torch.uint8, device="cuda")
    clips = torch.from_numpy(I.clips(N, T, S, 0, "bf16")).to(torch.bfloat16).cuda()      # N distinct clips
    params = torch.from_numpy(flat).cuda()
    # running statistics: mean 0, variance 1 (their values do not change the work done)
    state = np.concatenate([np.concatenate([np.zeros(sh[0]), np.ones(sh[0])]) for n, _, sh, _ in table if n.endswith(".g")])
    bn_state = torch.from_numpy(state.astype(np.float32)).cuda()
    logits = torch.empty((N, K), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def eager():
        B.tsm_resnet50_infer(d, clips, params, bn_state, logits, ws, torch.cuda.current_stream())

    step = eager
    if args.graph:      # the call is stream-ordered and allocates nothing: record it once, replay it per step
        eager()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            eager()
        step = graph.replay
    for _ in range(args.warmup):
        step()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record(stream)
    for _ in range(args.steps):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    if not bool(torch.isfinite(logits).all()):
        sys.exit("bench.py: logits are not finite")
    B.tsm_profile_begin(stream)
    eager()
    prof = B.tsm_profile_end()
    F = N * T
    work, byt = {}, {}
    fused_on = os.environ.get("TSM_FUSED_TAIL", "1")[:1] != "0"
    for name, rin, cin, rout, cout, taps, _ in conv_layers(F, S):
        stem = name == "conv1"
        cls = igemm_class("fwd", cout, 64 if stem else cin, rout, taps, "stem" if stem else (1 if rin == rout else 2), affine=True)
        x_b = 2.0 * F * (S // 2 + 3) ** 2 * 16 if stem else 2.0 * rin * cin
        res_b = 2.0 * rout * cout if name.endswith(".c3") else 0.0     # the shortcut read by the epilogue
        y_b = 2.0 * rout * cout
        # the 3x3 and the last 1x1 convolution of a bottleneck with 64 / 128 middle channels run as one kernel from
        # three quarters of a round of 256-pixel tiles on: the tensor between them is neither written nor read
        mid = cin if name.endswith(".c3") else cout
        if fused_on and name.endswith((".c2", ".c3")) and mid in (64, 128) and -(-rout // 256) >= 192:
            cls = "fused_tail_%d" % mid
            if name.endswith(".c2"):
                y_b = 0.0
            else:
                x_b = 0.0
        work[cls] = work.get(cls, 0.0) + 2.0 * rout * cout * cin * taps
        byt[cls] = byt.get(cls, 0.0) + x_b + y_b + res_b
    dom = max(prof, key=lambda k: prof[k][1])
    n_launch, dom_ms = prof[dom]
    roof = {"bound": "hbm", "kernel": dom, "launches_per_step": n_launch, "avg_launch_ms": dom_ms / n_launch,
            "achieved": None, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": None, "traffic": None}
    if dom in work:
        tflops, gbs = work[dom] / (dom_ms * 1e-3) / 1e12, byt[dom] / (dom_ms * 1e-3) / 1e9
        hbm_bound = byt[dom] / (PEAK_HBM_GBS * 1e9) > work[dom] / (PEAK_BF16_TFLOPS * 1e12)
        roof.update({"bound": "hbm" if hbm_bound else "mfma", "achieved": gbs if hbm_bound else tflops,
                     "peak": PEAK_HBM_GBS if hbm_bound else PEAK_BF16_TFLOPS, "unit": "GB/s" if hbm_bound else "TFLOP/s",
                     "frac": gbs / PEAK_HBM_GBS if hbm_bound else tflops / PEAK_BF16_TFLOPS,
                     "flops_per_launch": work[dom] / n_launch, "algorithmic_bytes_per_launch": byt[dom] / n_launch,
                     "tflops": tflops, "algorithmic_gbs": gbs})
    flops = sum(work.values())
    out = {"metric": "TSM-ResNet-50 inference videos/s (8x224^2, forward only, batch %d) at 1 GPU" % N,
           "value": N / (ms * 1e-3), "unit": "videos/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
           # the paper's figure for this workload (84.8 videos/s, batch 16) is one Tesla P100's: context, not a target
           "vs_baseline": (N / (ms * 1e-3) / 84.8) if N == 16 else None,
           "dtype": "bf16", "data": "synthetic",
           "config": {"workload": "Table 1 efficiency row: TSM-ResNet-50 forward only, %d clips x 8 frames x 3x224x224, "
                                  "400 classes, fold_div 8, BatchNorm with running statistics" % N,
                      "clips_per_step": N, "frames": T, "size": S, "num_classes": K},
           "step_tflops": flops / (ms * 1e-3) / 1e12,
           "pct_bf16_mfma_peak": 100.0 * flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
           "roofline": roof, "hip_graph": bool(args.graph),
           "kernel_classes": {k: {"launches": v[0], "ms": round(v[1], 4),
                                  "tflops": round(work[k] / (v[1] * 1e-3) / 1e12, 1) if k in work else None}
                              for k, v in sorted(prof.items(), key=lambda kv: -kv[1][1])},
           "profiled_step_ms": sum(v[1] for v in prof.values())}
    if not args.no_cpu_baseline:
        from oracle import tsm_oracle as O
        P = O.unflatten_params(flat.astype(np.float64))
        nc = 2
        c1 = I.clips(nc, T, S, 0, "bf16").astype(np.float64)
        t0 = time.perf_counter()
        O.resnet50_infer(P, state, c1)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": nc / dt, "unit": "videos/s", "cores": O.max_threads(), "kind": "oracle",
                               "sample": "%d clips of the same shape through the fp64 oracle's inference forward" % nc}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--clips", type=int, default=None,
                    help="clips per step: 64 = configs[3] (throughput run, the default), 8 = configs[2]; "
                         "--workload infer defaults to the paper's batch of 16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-overlap", action="store_true",
                    help="keep the weight gradients on the launch stream (the library otherwise runs them on a second "
                         "stream beside the data gradients); for per-kernel profiles with exclusive durations")
    ap.add_argument("--graph", action="store_true",
                    help="record one call into a HIP graph and time replays of it (step and infer workloads)")
    ap.add_argument("--workload", default="step", choices=["step", "res2", "cmp", "infer"],
                    help="step: the full train step (the headline, default); res2: configs[1], the three res2 bottlenecks "
                         "fwd+bwd at 8 clips; cmp: configs[4], TSM block against the 3x1x1 temporal-conv block")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (no collectives, no sharding); --gpus %d is not supported"
                 % args.gpus)

    if args.no_overlap:
        os.environ["TSM_WGRAD_OVERLAP"] = "0"      # read by the library when it first runs a block backward
    import torch
    from paper_1910_00932_amd import binding as B
    from paper_1910_00932_amd import inputs as I

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    if args.clips is None:
        args.clips = 16 if args.workload == "infer" else 64
    if args.workload == "infer":
        print(json.dumps(infer_workload(args, torch, B, I)))
        return
    if args.workload != "step":
        print(json.dumps(block_workload(args, torch, B, I)))
        return
    N, T, S, K = args.clips, 8, 224, 400
    lr = 0.00125 * N / 8.0          # linear scaling rule (paper section 4.1)
    table = B.tsm_resnet50_param_table(K)
    flat = I.init_params([(n, s) for n, _, s, _ in table], 1)
    d = B.R50Desc(N=N, T=T, size=S, num_classes=K, fold_div=8, lr=lr, momentum=0.9, weight_decay=1e-4, bn_eps=1e-5,
                  bn_momentum=0.1, dtype=B.TSM_BF16)
    ws_bytes = B.tsm_resnet50_workspace_bytes(d)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    # inputs are generated once and live in HBM before the timed region
    rng = np.random.default_rng(0)
    clips = torch.from_numpy(I.clips(N, T, S, 0, "bf16")).to(torch.bfloat16).cuda()      # N distinct clips
    labels = torch.from_numpy(I.labels(N, K)).cuda()
    params = torch.from_numpy(flat).cuda()
    mom = torch.zeros_like(params)
    bn_state = torch.zeros(B.tsm_resnet50_bn_state_count(), dtype=torch.float32, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def eager():
        B.tsm_resnet50_step(d, clips, labels, params, mom, bn_state, None, loss, None, 1, ws, torch.cuda.current_stream())

    step = eager
    if args.graph:      # the call is stream-ordered and allocates nothing: record it once, replay it per step
        eager()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            eager()
        step = graph.replay
    first_loss = None
    for i in range(args.warmup):
        step()
        if i == 0:
            torch.cuda.synchronize()
            first_loss = float(loss.item())      # the loss of the untrained network on this batch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    # one event per step boundary: the mean comes from the first and the last, median and minimum from the rest
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    ev[0].record(stream)
    for i in range(args.steps):
        step()
        ev[i + 1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = ev[0].elapsed_time(ev[-1]) / args.steps
    per_step = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(args.steps))
    final_loss = float(loss.item())
    if not np.isfinite(final_loss):
        sys.exit("bench.py: loss is not finite (%r)" % final_loss)
    # the steps train on one fixed batch: the loss the last step reports must lie below the untrained network's
    if first_loss is not None and not final_loss < first_loss:
        sys.exit("bench.py: the loss did not fall over %d steps on a fixed batch (%r -> %r)"
                 % (args.warmup + args.steps, first_loss, final_loss))

    # per-class time of one more step, HIP events on the launch stream after every launch
    B.tsm_profile_begin(stream)
    eager()
    prof = B.tsm_profile_end()
    work = class_work(N * T, S)
    ew_bytes = elementwise_bytes(N * T, S)
    traffic = measured_traffic(N)

    def class_roofline(dom):
        n_launch, dom_ms = prof[dom]
        if dom in work:
            return conv_roofline(dom, n_launch, dom_ms)
        if dom in ew_bytes:    # an elementwise pass: bytes at the HBM peak
            gbs = ew_bytes[dom] / (dom_ms * 1e-3) / 1e9
            return {"bound": "hbm", "kernel": dom, "launches_per_step": n_launch, "avg_launch_ms": dom_ms / n_launch,
                    "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                    "traffic": traffic.get(dom),
                    "traffic_source": "committed rocprofv3 --pmc summary under profiles/ (not measured in this run)"
                                      if traffic.get(dom) is not None else None,
                    "algorithmic_bytes_per_launch": ew_bytes[dom] / n_launch}
        return {"bound": "hbm", "kernel": dom, "launches_per_step": n_launch, "avg_launch_ms": dom_ms / n_launch,
                "achieved": None, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": None, "traffic": None}

    def conv_roofline(dom, n_launch, dom_ms):
        # the bound is the larger of the class's two floors: algorithmic FLOPs at the MFMA peak, algorithmic
        # bytes at the HBM peak
        tflops = work[dom] / (dom_ms * 1e-3) / 1e12
        alg_bytes = class_bytes(N * T, S)[dom]
        conv_bytes = class_bytes(N * T, S, epilogue_reads=False)[dom]
        gbs = alg_bytes / (dom_ms * 1e-3) / 1e9
        t_mfma, t_hbm = work[dom] / (PEAK_BF16_TFLOPS * 1e12), alg_bytes / (PEAK_HBM_GBS * 1e9)
        hbm_bound = t_hbm > t_mfma
        return {"bound": "hbm" if hbm_bound else "mfma", "kernel": dom, "launches_per_step": n_launch,
                "avg_launch_ms": dom_ms / n_launch,
                "achieved": gbs if hbm_bound else tflops, "peak": PEAK_HBM_GBS if hbm_bound else PEAK_BF16_TFLOPS,
                "unit": "GB/s" if hbm_bound else "TFLOP/s",
                "frac": (gbs / PEAK_HBM_GBS) if hbm_bound else (tflops / PEAK_BF16_TFLOPS),
                "traffic": traffic.get(dom),
                "traffic_source": "committed rocprofv3 --pmc summary under profiles/ (not measured in this run)"
                                  if traffic.get(dom) is not None else None,
                "flops_per_launch": work[dom] / n_launch, "algorithmic_bytes_per_launch": alg_bytes / n_launch,
                "tflops": tflops, "algorithmic_gbs": gbs,
                "frac_of_mfma_peak": tflops / PEAK_BF16_TFLOPS, "frac_of_hbm_peak": gbs / PEAK_HBM_GBS,
                # the same launches on two byte accountings: `frac` counts what the kernel has to move for the
                # method's work it carries (convolution operand and result, plus the shortcut gradient, ReLU-mask
                # source and BatchNorm input its fused epilogue reads); the second one counts the convolution's
                # operand and result alone
                "frac_conv_bytes_only": conv_bytes / (dom_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                "conv_bytes_per_launch": conv_bytes / n_launch}

    # the dominant class of the step, and (where that is an elementwise pass) the largest convolution class beside it
    roof = class_roofline(max(prof, key=lambda k: prof[k][1]))
    conv_dom = max((k for k in prof if k in work), key=lambda k: prof[k][1])
    roof_conv = class_roofline(conv_dom)
    prof_total = sum(v[1] for v in prof.values())
    classes = {k: {"launches": v[0], "ms": round(v[1], 4),
                   "tflops": round(work[k] / (v[1] * 1e-3) / 1e12, 1) if k in work else None}
               for k, v in sorted(prof.items(), key=lambda kv: -kv[1][1])}

    flops_step = sum(work.values())
    out = {
        "metric": "TSM-ResNet-50 train clips/sec (8x224^2, fwd+bwd) at 1 GPU; % bf16 MFMA peak",
        "value": N / (ms_per_step * 1e-3), "unit": "clips/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[%d]: full TSM-ResNet-50 train step, %d clips x 8 frames x 3x224x224, 400 classes, "
                               "fold_div 8, SGD momentum 0.9" % (3 if N == 64 else 2, N),
                   "clips_per_step": N, "frames": T, "size": S, "num_classes": K},
        "step_tflops": flops_step / (ms_per_step * 1e-3) / 1e12,
        "pct_bf16_mfma_peak": 100.0 * flops_step / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "ms_per_step_median": per_step[len(per_step) // 2], "ms_per_step_min": per_step[0],
        "loss_before": first_loss, "loss_after": final_loss, "wall_s": wall, "hip_graph": bool(args.graph), "wgrad_overlap": not args.no_overlap,
        "roofline": roof, "roofline_largest_conv_class": roof_conv, "kernel_classes": classes, "profiled_step_ms": prof_total,
    }

    # the stand-alone shift (a pure gather copy) at the configs[1] activation shape x 64 clips: HBM GB/s
    sh_shape = (64, 8, 256, 56, 56)
    nbytes = int(np.prod(sh_shape)) * 2
    xs = torch.empty(nbytes // 2, dtype=torch.bfloat16, device="cuda").normal_()
    ys = torch.empty_like(xs)
    for fn in (B.tsm_shift_fwd, B.tsm_shift_bwd):
        fn(xs, ys, *sh_shape, 8, B.TSM_BF16, B.TSM_NTHWC, stream)
    s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 20
    s0.record(stream)
    for _ in range(reps):
        B.tsm_shift_fwd(xs, ys, *sh_shape, 8, B.TSM_BF16, B.TSM_NTHWC, stream)
    s1.record(stream)
    torch.cuda.synchronize()
    sh_ms = s0.elapsed_time(s1) / reps
    sh_gbs = 2.0 * nbytes / (sh_ms * 1e-3) / 1e9
    # reference: the framework's own device-to-device copy of the same buffer (what a plain copy reaches here)
    ys.copy_(xs)
    s0.record(stream)
    for _ in range(reps):
        ys.copy_(xs)
    s1.record(stream)
    torch.cuda.synchronize()
    cp_gbs = 2.0 * nbytes / (s0.elapsed_time(s1) / reps * 1e-3) / 1e9
    out["shift"] = {"shape": list(sh_shape), "dtype": "bf16", "layout": "NTHWC", "ms": sh_ms, "achieved": sh_gbs,
                    "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": sh_gbs / PEAK_HBM_GBS,
                    "bytes": "one read + one write of the tensor", "plain_copy_gbs": cp_gbs}
    del xs, ys

    # what the matrix cores sustain with nothing in the way (register-only bf16 MFMAs), next to the published peak
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    B.tsm_mfma_probe(1000, sink, stream)
    s0.record(stream)
    probe_flops = B.tsm_mfma_probe(20000, sink, stream)
    s1.record(stream)
    torch.cuda.synchronize()
    out["mfma_probe"] = {"achieved": probe_flops / (s0.elapsed_time(s1) * 1e-3) / 1e12, "peak": PEAK_BF16_TFLOPS,
                         "unit": "TFLOP/s", "kernel": "register-only v_mfma_f32_32x32x16_bf16, 8 wavefronts per CU"}

    if not args.no_cpu_baseline:
        from oracle import tsm_oracle as O
        P = O.unflatten_params(flat.astype(np.float64))
        V = {k: np.zeros_like(v) for k, v in P.items()}
        nc = 2   # bounded sample: two clips keep the oracle's run to roughly ten seconds
        c1 = I.clips(nc, T, S, 0, "bf16").astype(np.float64)
        t0 = time.perf_counter()
        O.resnet50_step(P, V, c1, I.labels(nc, K), lr)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": nc / dt, "unit": "clips/s", "cores": O.max_threads(), "kind": "oracle",
                               "sample": "%d clips (8x3x224x224 each): one full fwd+bwd+update of the fp64 oracle, %.1f s"
                                         % (nc, dt)}
        # the same oracle on one thread, on a smaller sample of the same workload (one clip, forward pass only)
        nthreads = O.max_threads()
        O.set_threads(1)
        bn0 = np.concatenate([np.concatenate([np.zeros(sh[0]), np.ones(sh[0])]) for n, _, sh, _ in table if n.endswith(".g")])
        t0 = time.perf_counter()
        O.resnet50_infer(P, bn0, c1[:1])
        dt1 = time.perf_counter() - t0
        O.set_threads(nthreads)
        out["cpu_baseline_single_thread"] = {"value": 1.0 / dt1, "unit": "clips/s (forward only)", "cores": 1, "kind": "oracle",
                                             "sample": "1 clip (8x3x224x224): forward pass of the fp64 oracle on one thread, %.1f s" % dt1}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
