#!/usr/bin/env python3
"""Benchmark of the capsule-convolution forward pass on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5] [--path auto|mfma|direct]
                    [--op fwd|bwd_input|bwd_kernel|scheme1|scheme2|framework_conv|net5]

A step is one pass of the whole hot path (kernel repack, window addressing, LDS staging,
matrix-core contraction, accumulation, fp32 store) over one batch of seeded synthetic input
that is already resident in HBM.  The default workload is benchmark configuration 5
(fp16 in, fp32 accumulate, N=64, 32x32, C=M=64, 3x3, pad 1, 16x16 capsules), the largest one
and the one the roofline target is stated on.  `--op bwd_input` / `--op bwd_kernel` time the
backward pass (gradient with respect to the input / the kernel) of the same workload instead;
`--op scheme1|scheme2|framework_conv` time the comparison implementations of the forward pass
(the paper's two schemes and the framework's grouped convolution) on the same inputs.
`--op net5` times a five-layer stack of bf16 capsule convolutions chained through the
16-bit-output entry point (--config is ignored).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published dense peaks (TFLOP/s) and HBM bandwidth
PEAK_TFLOPS = {"fp32": 157.3, "bf16": 2516.6, "fp16": 2516.6}
PEAK_HBM_GBS = 8000.0
PEAK_ALU_TFLOPS = 78.6   # fp32 FMAs on the vector ALUs without the packed forms

# HBM-side bytes per launch of the dominant kernel come from profiles/hbm_traffic.json: rocprofv3
# --pmc FETCH_SIZE / WRITE_SIZE readings, scaled by a plain device copy of known size in the same
# process, recorded together with hashes of the kernel sources they were taken with.  A reading
# whose sources have changed since is not reported (null).
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")
KERNEL_SOURCES = {  # what the dominant kernel of each benchmark configuration is built from
    1: ["igemm_small.hip", "igemm_common.h", "conv_shape.h"],
    2: ["igemm32_dma.hip", "igemm_conv.hip", "igemm_common.h", "lds_dma.h", "conv_shape.h"],
    3: ["igemm16_fast.hip", "igemm_conv.hip", "igemm_common.h", "lds_dma.h", "conv_shape.h"],
    4: ["igemm_small.hip", "igemm_common.h", "conv_shape.h"],
    5: ["igemm16_fast.hip", "igemm_conv.hip", "igemm_common.h", "lds_dma.h", "conv_shape.h"],
}


def source_hashes(config):
    import hashlib
    csrc = os.path.join(ROOT, "paper_2104_02621_amd", "csrc")
    return {name: hashlib.sha256(open(os.path.join(csrc, name), "rb").read()).hexdigest()[:16]
            for name in KERNEL_SOURCES[config]}


def measured_traffic_bytes(config):
    """Bytes past the L2s per launch of the configuration's dominant kernel, or None when no
    reading exists for the kernel sources as they are now."""
    try:
        entries = json.load(open(TRAFFIC_FILE))["entries"]
    except (OSError, ValueError, KeyError):
        return None
    for e in entries:
        if e.get("config") == config and e.get("sources") == source_hashes(config):
            return int((e["fetch_kib"] * e["fetch_scale"] + e["write_kib"] * e["write_scale"]) * 1024)
    return None


def record_traffic(config, fetch_dir, write_dir):
    """Reads the counter_collection.csv files of two rocprofv3 --pmc runs of
    `bench.py --config N --copy-probe` (FETCH_SIZE in one, WRITE_SIZE in the other) and writes
    the configuration's entry of profiles/hbm_traffic.json."""
    import csv
    import glob
    import subprocess

    def read(directory, counter):
        files = glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True)
        if not files:
            sys.exit(f"bench.py: no counter_collection.csv under {directory}")
        per_kernel = {}
        for row in csv.DictReader(open(files[0])):
            if row["Counter_Name"] == counter:
                per_kernel.setdefault(row["Kernel_Name"], []).append(float(row["Counter_Value"]))
        copies = [v for k, vs in per_kernel.items() if "copyBuffer" in k for v in vs]
        ours = {k: sum(vs) / len(vs) for k, vs in per_kernel.items() if "capscaps" in k}
        if not copies or not ours:
            sys.exit(f"bench.py: {directory} holds no copy kernel or no capscaps kernel")
        return max(copies), ours

    fetch_copy, fetch = read(fetch_dir, "FETCH_SIZE")
    write_copy, write = read(write_dir, "WRITE_SIZE")
    kernel = max(fetch, key=lambda k: fetch[k] + write.get(k, 0.0))
    # --copy-probe copies 1 GiB; the runtime may cut it into equal dispatches, so the largest
    # dispatch's WRITE_SIZE tells its size, and FETCH_SIZE of the same dispatch reads that size
    probe_kib = float(1 << 20)
    pieces = max(1, round(probe_kib / write_copy))
    entry = {
        "config": config,
        "kernel": kernel.replace("(anonymous namespace)::", "").replace("capscaps::", "")
                        .replace("void ", "").split("(")[0][:80],
        "fetch_kib": round(fetch[kernel], 1), "write_kib": round(write.get(kernel, 0.0), 1),
        "fetch_scale": round(probe_kib / pieces / fetch_copy, 4),
        "write_scale": round(probe_kib / pieces / write_copy, 4),
        "sources": source_hashes(config),
        "command": (f"rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE --output-format csv -d <dir> -o r -- python3 "
                    f"bench.py --config {config} --steps 3 --warmup 1 --no-cpu-baseline --no-yardstick "
                    f"--copy-probe; python3 bench.py --config {config} --record-traffic <fetch dir> <write dir>"),
    }
    try:
        entry["commit"] = subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"],
                                         capture_output=True, text=True).stdout.strip() or None
    except OSError:
        entry["commit"] = None
    try:
        data = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        data = {"what": "HBM-side bytes per launch of each configuration's dominant kernel "
                        "(rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, KiB per dispatch, scaled by a "
                        "1 GiB device copy in the same process); read by bench.py",
                "entries": []}
    data["entries"] = [e for e in data["entries"] if e.get("config") != config] + [entry]
    data["entries"].sort(key=lambda e: e["config"])
    json.dump(data, open(TRAFFIC_FILE, "w"), indent=1)
    print(json.dumps(entry))


def cpu_baseline(w, i32, k32, gpu_out, target_seconds=15.0):
    """Times the oracle, as it stands, on a bounded sample of the same workload, and uses the
    sample to check the GPU result.  Returns (record, max error relative to max |ref|)."""
    import numpy as np
    from oracle import capsconv
    from paper_2104_02621_amd import workloads as wl

    flops_per_capsule = 2 * w.D0 * w.D1 * w.D3 * w.kh * w.kw * w.C * w.D2
    probe = wl.sample_capsules(w, 64, seed=4242)
    t0 = time.perf_counter()
    capsconv.conv_fwd_subset(i32, k32, probe, w.stride, w.pad)
    dt = max(time.perf_counter() - t0, 1e-4)
    total = w.N * w.Ho * w.Wo * w.M
    count = int(min(total, max(64, 64 * target_seconds / dt)))
    which = wl.sample_capsules(w, count, seed=4243)
    t0 = time.perf_counter()
    ref = capsconv.conv_fwd_subset(i32, k32, which, w.stride, w.pad)
    dt = time.perf_counter() - t0
    gflops = count * flops_per_capsule / dt / 1e9
    import torch
    idx = torch.from_numpy(which.astype(np.int64)).to(gpu_out.device)
    got = gpu_out[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]].cpu().numpy()
    err = float(np.abs(got - ref).max() / np.abs(ref).max())
    rec = {
        "value": round(gflops, 3), "unit": "GFLOP/s", "cores": capsconv.threads(),
        "kind": "oracle",
        "sample": (f"{count} of {total} output capsules (n,x,y,m) of the same workload, fixed "
                   f"seed, 25% on image borders; {dt:.1f} s; nominal FLOPs of the sample; "
                   f"full workload extrapolates to {w.flops_nominal() / gflops / 1e9:.0f} s"),
    }
    return rec, err


def cpu_baseline_bwd(w, op, i32, k32, g32, gpu_grad, target_seconds=12.0):
    """Backward counterpart: the oracle on slices it can compute exactly from sliced operands
    (dI[n,:,:,c] from image n of the gradient and channel c of the kernel; dK[:,:,c,m] from
    channel c of the input and channel m of the gradient)."""
    import numpy as np
    from oracle import capsconv

    rng = np.random.default_rng(4244)
    op = "bwd_input" if op == "bwd_input_out16" else op
    slices = w.N * w.C if op == "bwd_input" else w.C * w.M
    flops_per_slice = w.flops_tap_exact() / slices
    done, spent, err, ref_max = 0, 0.0, 0.0, 0.0
    while done < slices and (done == 0 or spent * (done + 1) / done < target_seconds):
        if op == "bwd_input":
            n, c = int(rng.integers(w.N)), int(rng.integers(w.C))
            a, b = g32[n:n + 1], np.ascontiguousarray(k32[:, :, c:c + 1])
            t0 = time.perf_counter()
            ref = capsconv.conv_bwd_input(a, b, (w.H, w.W), w.stride, w.pad)
            spent += time.perf_counter() - t0
            got = gpu_grad[n:n + 1, :, :, c:c + 1].float().cpu().numpy()
        else:
            c, m = int(rng.integers(w.C)), int(rng.integers(w.M))
            a = np.ascontiguousarray(i32[:, :, :, c:c + 1])
            b = np.ascontiguousarray(g32[:, :, :, m:m + 1])
            t0 = time.perf_counter()
            ref = capsconv.conv_bwd_kernel(a, b, (w.kh, w.kw), w.stride, w.pad)
            spent += time.perf_counter() - t0
            got = gpu_grad[:, :, c:c + 1, m:m + 1].cpu().numpy()
        err = max(err, float(np.abs(got - ref).max()))
        ref_max = max(ref_max, float(np.abs(ref).max()))
        done += 1
    gflops = done * flops_per_slice / spent / 1e9
    what = "dI[n,:,:,c]" if op == "bwd_input" else "dK[:,:,c,m]"
    rec = {
        "value": round(gflops, 3), "unit": "GFLOP/s", "cores": capsconv.threads(),
        "kind": "oracle",
        "sample": (f"{done} of {slices} slices {what} of the same workload, fixed seed; "
                   f"{spent:.1f} s; tap-exact FLOPs of the sample; full workload extrapolates "
                   f"to {w.flops_tap_exact() / gflops / 1e9:.0f} s"),
    }
    return rec, err / max(ref_max, 1e-300)


def mfma_yardstick(dtype, zero_data=False, seconds=0.05):
    """Sustained rate (TFLOP/s) of back-to-back matrix instructions on register operands, with
    N(0,1) operands (or zeros), 1024 workgroups.  Timed with events on torch's current stream."""
    import numpy as np
    import torch
    from paper_2104_02621_amd import capscaps as cc
    from paper_2104_02621_amd import workloads as wl

    rng = np.random.default_rng(31337)
    n_elem = 8 * 64 * (4 if dtype == wl.FP32 else 8)
    vals = np.zeros(n_elem, dtype=np.float32) if zero_data else \
        rng.standard_normal(n_elem).astype(np.float32)
    st, _ = wl.to_storage(vals, dtype)
    seed = torch.from_numpy(st.view(np.int16) if dtype == wl.BF16 else st).cuda()
    blocks = 1024
    sink = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def run(iters):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        rc = cc.capscaps_mfma_yardstick(seed.data_ptr(), sink.data_ptr(), dtype, blocks, iters,
                                        stream.cuda_stream)
        e1.record(stream)
        torch.cuda.synchronize()
        if rc != cc.OK:
            sys.exit(f"bench.py: yardstick status {rc}")
        return e0.elapsed_time(e1) * 1e-3

    t = run(200)
    iters = int(min(1 << 22, max(200, 200 * seconds / max(t, 1e-6))))
    run(iters)                       # settle the clocks under load
    t = min(run(iters) for _ in range(3))
    return cc.capscaps_mfma_yardstick_flops(dtype, blocks, iters) / t / 1e12


def bench_net5(args):
    """Five chained layers (workloads.net5): layers 1-4 write bf16 activations that the next layer
    reads as they are, layer 5 writes fp32.  One step = the five calls.  With --op net5_train a
    step is a forward and a backward pass, the two columns of the paper's Table 1: top down, every
    layer's kernel gradient (fp32) and, for layers 5..2, its input gradient in bf16, which is the
    output gradient of the layer below (layer 1's input gradient is of no use to training and is
    not computed); the last layer's output gradient is a seeded bf16 tensor."""
    import numpy as np
    import torch
    from oracle import capsconv
    from paper_2104_02621_amd import capscaps as cc
    from paper_2104_02621_amd import workloads as wl

    torch.cuda.set_device(0)
    layers = wl.net5(N=64)
    i_st, _, i32, _ = wl.generate(layers[0])
    x0 = torch.from_numpy(i_st.view(np.int16)).cuda().view(torch.bfloat16)
    kernels32 = [wl.generate(w)[3] for w in layers]
    kernels = [torch.from_numpy(wl.generate(w)[1].view(np.int16)).cuda().view(torch.bfloat16)
               for w in layers]
    stream = torch.cuda.current_stream()
    outs, wss, shapes = [], [], []
    for k, w in enumerate(layers):
        last = k + 1 == len(layers)
        shape = (w.N, w.H, w.W, w.C, w.M, w.kh, w.kw, w.stride, w.pad, w.D0, w.D1, w.D2, w.D3,
                 w.dtype)
        need = (cc.capscaps_conv_fwd_workspace_bytes if last else
                cc.capscaps_conv_fwd_out16_workspace_bytes)(*shape)
        outs.append(torch.empty(w.out_shape, dtype=torch.float32 if last else torch.bfloat16,
                                device="cuda"))
        wss.append(torch.empty(max(need, 16), dtype=torch.uint8, device="cuda"))
        shapes.append(shape)
    train = args.op == "net5_train"
    if train:
        g_top = torch.from_numpy(wl.generate_dout(layers[-1])[0].view(np.int16)).cuda().view(torch.bfloat16)
        # gin[k]: gradient with respect to layer k's input = output gradient of layer k-1
        gin = [None] + [torch.empty(w.input_shape, dtype=torch.bfloat16, device="cuda")
                        for w in layers[1:]]
        dks = [torch.empty(w.kernel_shape, dtype=torch.float32, device="cuda") for w in layers]
        need = max(max(cc.capscaps_conv_bwd_kernel_workspace_bytes(*s) for s in shapes),
                   max(cc.capscaps_conv_bwd_input_out16_workspace_bytes(*s) for s in shapes[1:]))
        ws_bwd = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")

    def forward():
        x = x0
        for k in range(len(layers)):
            fn = cc.capscaps_conv_fwd_ex if k + 1 == len(layers) else cc.capscaps_conv_fwd_out16
            rc = fn(x.data_ptr(), kernels[k].data_ptr(), outs[k].data_ptr(), *shapes[k],
                    wss[k].data_ptr(), wss[k].numel(), stream.cuda_stream)
            if rc != cc.OK:
                sys.exit(f"bench.py: capscaps status {rc}: {cc.capscaps_strerror(rc)}")
            x = outs[k]

    def backward():
        g = g_top
        for k in range(len(layers) - 1, -1, -1):
            x = x0 if k == 0 else outs[k - 1]
            rc = cc.capscaps_conv_bwd_kernel(x.data_ptr(), g.data_ptr(), dks[k].data_ptr(),
                                             *shapes[k], ws_bwd.data_ptr(), ws_bwd.numel(),
                                             stream.cuda_stream)
            if rc == cc.OK and k > 0:
                rc = cc.capscaps_conv_bwd_input_out16(g.data_ptr(), kernels[k].data_ptr(),
                                                      gin[k].data_ptr(), *shapes[k],
                                                      ws_bwd.data_ptr(), ws_bwd.numel(),
                                                      stream.cuda_stream)
                g = gin[k]
            if rc != cc.OK:
                sys.exit(f"bench.py: capscaps status {rc}: {cc.capscaps_strerror(rc)}")

    fwd_ms = []

    def step():
        forward()
        if train:
            mid_ev = torch.cuda.Event(enable_timing=True)
            mid_ev.record(stream)
            fwd_ms.append(mid_ev)
            backward()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    ev[0].record(stream)
    for k in range(args.steps):
        step()
        ev[k + 1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    kernel_ms = float(np.mean([ev[k].elapsed_time(ev[k + 1]) for k in range(args.steps)]))
    flops = sum(w.flops_tap_exact() for w in layers)
    fwd_flops = flops
    if train:  # each gradient has the forward pass's terms; layer 1's input gradient is left out
        flops = 3 * flops - layers[0].flops_tap_exact()
        mids = fwd_ms[-args.steps:]
        forward_ms = float(np.mean([ev[k].elapsed_time(mids[k]) for k in range(args.steps)]))
    achieved = flops / (kernel_ms * 1e-3) / 1e12
    result = {
        "metric": ("capsule-conv net5 forward + backward useful GFLOP/s at 1 GPU" if train else
                   "capsule-conv net5 useful GFLOP/s at 1 GPU"),
        "value": round(flops / (ms_per_step * 1e-3) / 1e9, 1), "unit": "GFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 in, f32 accumulate, bf16 activations", "data": "synthetic",
        "config": {"workload": "net5: five chained capsule convolutions, 8x8 capsules, N=64, 32x32",
                   "op": args.op, "layers": [w.name + " " + "x".join(map(str, w.out_shape))
                                             for w in layers],
                   "flops_tap_exact": flops},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_TFLOPS["bf16"],
                     "unit": "TFLOP/s", "frac": round(achieved / PEAK_TFLOPS["bf16"], 4),
                     "traffic": None, "kernel_ms": round(kernel_ms, 4)},
    }
    if train:
        result["config"]["forward_ms"] = round(forward_ms, 4)
        result["config"]["backward_ms"] = round(kernel_ms - forward_ms, 4)
    if not args.no_cpu_baseline:
        # the oracle on image 0 through all five layers, activations rounded as on the GPU
        x32 = i32[:1]
        t0 = time.perf_counter()
        for k, w in enumerate(layers):
            y = capsconv.conv_fwd(x32, kernels32[k], w.stride, w.pad)
            if k + 1 < len(layers):
                x32 = wl.to_storage(y.astype(np.float32), w.dtype)[1]
        dt = time.perf_counter() - t0
        got = outs[-1][:1].cpu().numpy()
        result["cpu_baseline"] = {
            "value": round(fwd_flops / 64 / dt / 1e9, 3), "unit": "GFLOP/s",
            "cores": capsconv.threads(), "kind": "oracle",
            "sample": f"image 0 of 64 through all five layers, forward; {dt:.1f} s"}
        result["config"]["max_err_vs_oracle_sample"] = float(np.abs(got - y).max() / np.abs(y).max())
    print(json.dumps(result), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=5, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--path", default="auto",
                    choices=["auto", "mfma", "direct", "mfma-generic", "mfma-tuned16", "mfma-tuned32",
                             "mfma-small"])
    ap.add_argument("--op", default="fwd", choices=["fwd", "bwd_input", "bwd_input_out16", "bwd_kernel",
                                                     "scheme1", "scheme2", "framework_conv", "net5", "net5_train"])
    ap.add_argument("--shape", default=None,
                    help="N,H,W,C,M,kh,kw,stride,pad,D0,D1,D2,D3: time this layer instead of a "
                         "benchmark configuration (inputs N(0,1), kernel N(0, 1/fan-in); --dtype)")
    ap.add_argument("--dtype", default="fp32", choices=["fp32", "bf16", "fp16"],
                    help="element type for --shape")
    ap.add_argument("--record-traffic", nargs=2, metavar=("FETCH_DIR", "WRITE_DIR"), default=None,
                    help="no GPU work: read two rocprofv3 --pmc outputs (FETCH_SIZE, WRITE_SIZE) of "
                         "`bench.py --config N --copy-probe` and write N's entry of "
                         "profiles/hbm_traffic.json")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step (all its launches) in a HIP graph and time replays; for "
                         "the launch-bound small configurations")
    ap.add_argument("--no-yardstick", action="store_true",
                    help="skip the register-resident MFMA loop that measures the sustained rate")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB device copy (the known-size kernel that "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings are scaled by)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build measures the capsule convolution on ONE GPU only "
                 "(the forward pass shards over the batch with no exchange step); run with --gpus 1")

    if args.record_traffic:
        return record_traffic(args.config, *args.record_traffic)

    import numpy as np
    import torch
    from paper_2104_02621_amd import capscaps as cc
    from paper_2104_02621_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    if args.op in ("net5", "net5_train"):
        return bench_net5(args)
    torch.cuda.set_device(0)
    w = wl.config(args.config)
    if args.shape:
        dims = [int(v) for v in args.shape.split(",")]
        if len(dims) != 13:
            sys.exit("bench.py: --shape takes 13 comma-separated integers")
        N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3 = dims
        dt = {"fp32": wl.FP32, "bf16": wl.BF16, "fp16": wl.FP16}[args.dtype]
        w = wl.Workload("shape_" + args.shape.replace(",", "_"), dt, N, H, W, C, M, kh, kw, stride,
                        pad, D0, D1, D2, D3, "normal", "normal",
                        1.0 / float(np.sqrt(kh * kw * C * D2)), 7001, 7002)
    path = {"auto": cc.PATH_AUTO, "mfma": cc.PATH_MFMA, "direct": cc.PATH_DIRECT,
            "mfma-generic": cc.PATH_MFMA_GENERIC, "mfma-tuned16": cc.PATH_MFMA_TUNED16,
            "mfma-tuned32": cc.PATH_MFMA_TUNED32, "mfma-small": cc.PATH_MFMA_SMALL}[args.path]
    shape = (w.N, w.H, w.W, w.C, w.M, w.kh, w.kw, w.stride, w.pad, w.D0, w.D1, w.D2, w.D3, w.dtype)

    i_st, k_st, i32, k32 = wl.generate(w)
    if w.dtype == wl.BF16:
        I = torch.from_numpy(i_st.view(np.int16)).cuda().view(torch.bfloat16)
        K = torch.from_numpy(k_st.view(np.int16)).cuda().view(torch.bfloat16)
    else:
        I = torch.from_numpy(i_st).cuda()
        K = torch.from_numpy(k_st).cuda()
    g32 = None
    comparison = args.op in ("scheme1", "scheme2", "framework_conv")
    if args.op == "fwd":
        out = torch.empty(w.out_shape, dtype=torch.float32, device="cuda")
        need = cc.capscaps_conv_fwd_workspace_bytes(*shape)
    elif comparison:
        if args.path != "auto":
            sys.exit("bench.py: --path applies to --op fwd only")
        from paper_2104_02621_amd import comparisons as cmp
        out = torch.empty(w.out_shape, dtype=torch.float32, device="cuda")
        need = 0
        if args.op == "scheme1" and w.M * w.kh * w.kw * w.C * w.D0 > cmp.MAX_BMM_BATCH:
            sys.exit("bench.py: scheme 1 is not run on this workload (more small products per "
                     "output pixel than one batched multiply is handed; see "
                     "comparisons.MAX_BMM_BATCH)")
        if args.op == "scheme2":
            need = cc.capscaps_scheme2_index_bytes(*shape)
            if need == 0 or need > (64 << 30):
                sys.exit("bench.py: scheme 2's index arrays do not fit for this workload")
    else:
        if args.path != "auto":
            sys.exit("bench.py: --path applies to --op fwd only")
        g_st, g32 = wl.generate_dout(w)
        G = (torch.from_numpy(g_st.view(np.int16)).cuda().view(torch.bfloat16)
             if w.dtype == wl.BF16 else torch.from_numpy(g_st).cuda())
        if args.op == "bwd_input":
            out = torch.empty(w.input_shape, dtype=torch.float32, device="cuda")
            need = cc.capscaps_conv_bwd_input_workspace_bytes(*shape)
        elif args.op == "bwd_input_out16":
            if w.dtype == wl.FP32:
                sys.exit("bench.py: --op bwd_input_out16 needs a 16-bit workload")
            out = torch.empty(w.input_shape, device="cuda",
                              dtype=torch.bfloat16 if w.dtype == wl.BF16 else torch.float16)
            need = cc.capscaps_conv_bwd_input_out16_workspace_bytes(*shape)
        else:
            out = torch.empty(w.kernel_shape, dtype=torch.float32, device="cuda")
            need = cc.capscaps_conv_bwd_kernel_workspace_bytes(*shape)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    if args.op == "scheme2":  # the index arrays depend on the shape only: built once, untimed
        rc = cc.capscaps_scheme2_build_index(ws.data_ptr(), ws.numel(), *shape, stream.cuda_stream)
        if rc != cc.OK:
            sys.exit(f"bench.py: capscaps status {rc}: {cc.capscaps_strerror(rc)}")

    def step():
        if args.op == "fwd":
            rc = cc.capscaps_conv_fwd_path(I.data_ptr(), K.data_ptr(), out.data_ptr(),
                                           *shape[:13], w.dtype, path, ws.data_ptr(), ws.numel(),
                                           stream.cuda_stream)
        elif args.op == "scheme1":
            out.copy_(cmp.scheme1_fwd(I, K, w.stride, w.pad))
            return
        elif args.op == "framework_conv":
            out.copy_(cmp.framework_conv_fwd(I, K, w.stride, w.pad, widen=False))
            return
        elif args.op == "scheme2":
            rc = cc.capscaps_scheme2_fwd(I.data_ptr(), K.data_ptr(), out.data_ptr(), ws.data_ptr(),
                                         ws.numel(), *shape, stream.cuda_stream)
        elif args.op == "bwd_input":
            rc = cc.capscaps_conv_bwd_input(G.data_ptr(), K.data_ptr(), out.data_ptr(), *shape,
                                            ws.data_ptr(), ws.numel(), stream.cuda_stream)
        elif args.op == "bwd_input_out16":
            rc = cc.capscaps_conv_bwd_input_out16(G.data_ptr(), K.data_ptr(), out.data_ptr(), *shape,
                                                  ws.data_ptr(), ws.numel(), stream.cuda_stream)
        else:
            rc = cc.capscaps_conv_bwd_kernel(I.data_ptr(), G.data_ptr(), out.data_ptr(), *shape,
                                             ws.data_ptr(), ws.numel(), stream.cuda_stream)
        if rc != cc.OK:
            sys.exit(f"bench.py: capscaps status {rc}: {cc.capscaps_strerror(rc)}")

    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")   # 1 GiB
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    run_step = step
    if args.graph:
        # the library's calls only enqueue kernels on the stream they are given (no allocation,
        # no memset, no synchronisation), so a step can be captured and replayed as one graph
        eager = out.clone()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            stream = torch.cuda.current_stream()
            with torch.cuda.graph(graph, stream=side):
                step()
        stream = torch.cuda.current_stream()
        for _ in range(3):   # replays must reproduce the eager result every time
            out.zero_()
            graph.replay()
            torch.cuda.synchronize()
            if not torch.equal(out, eager):
                sys.exit("bench.py: graph replay differs from the eager result")
        run_step = graph.replay
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    ev[0].record(stream)
    for k in range(args.steps):
        run_step()
        ev[k + 1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per_step_ms = [ev[k].elapsed_time(ev[k + 1]) for k in range(args.steps)]
    ms_per_step = wall * 1e3 / args.steps
    kernel_ms = float(np.mean(per_step_ms))  # HIP events on the launch stream, per step

    flops_exact = w.flops_tap_exact()
    flops_nominal = w.flops_nominal()
    value = flops_exact / (ms_per_step * 1e-3) / 1e9
    dname = wl.DTYPE_NAMES[w.dtype]
    achieved_tflops = flops_exact / (kernel_ms * 1e-3) / 1e12
    chosen = cc.capscaps_select_path(*shape) if path in (cc.PATH_AUTO, cc.PATH_MFMA) else path
    result = {
        "metric": ("capsule-conv useful GFLOP/s at 1 GPU + % of MFMA roofline" if args.op == "fwd"
                   else f"capsule-conv {args.op} useful GFLOP/s at 1 GPU"),
        "value": round(value, 1), "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32" if w.dtype == wl.FP32 else
        f"{dname} in, f32 accumulate", "data": "synthetic",
        "config": {
            "workload": w.name if args.shape else f"config {args.config}: {w.name}", "op": args.op,
            "launch": "hip graph replay" if args.graph else "eager", "N": w.N, "H": w.H, "W": w.W, "C": w.C,
            "M": w.M, "kh": w.kh, "kw": w.kw, "stride": w.stride, "pad": w.pad,
            "capsule": [w.D0, w.D1, w.D2, w.D3],
            "path": {1: "direct", 2: "mfma", 3: "mfma-generic", 4: "mfma-tuned16",
                     5: "mfma-tuned32", 6: "mfma-small"}[chosen] if args.op == "fwd" else "auto",
            "flops_tap_exact": flops_exact, "flops_nominal": flops_nominal,
            "gflops_nominal": round(flops_nominal / (ms_per_step * 1e-3) / 1e9, 1),
            "compulsory_bytes": w.compulsory_bytes(),
            "hbm_gbs_compulsory": round(w.compulsory_bytes() / (kernel_ms * 1e-3) / 1e9, 1),
            "pct_of_mfma_peak": round(100 * achieved_tflops / PEAK_TFLOPS[dname], 2),
            "ms_min": round(float(np.min(per_step_ms)), 4),
            "ms_median": round(float(np.median(per_step_ms)), 4),
        },
        "roofline": {
            # the wavefront-level path is plain fp32 FMAs on the vector ALUs: 256 CUs x 4 SIMDs x
            # 16 lanes x 2 FLOP x 2.4 GHz (packed-fp32 forms are not used)
            "bound": "alu" if chosen == cc.PATH_DIRECT and args.op == "fwd" else "mfma",
            "achieved": round(achieved_tflops, 2),
            "peak": PEAK_ALU_TFLOPS if chosen == cc.PATH_DIRECT and args.op == "fwd" else PEAK_TFLOPS[dname],
            "unit": "TFLOP/s",
            "frac": round(achieved_tflops / (PEAK_ALU_TFLOPS if chosen == cc.PATH_DIRECT and
                                             args.op == "fwd" else PEAK_TFLOPS[dname]), 4),
            "traffic": (measured_traffic_bytes(args.config)
                        if args.op == "fwd" and not args.shape and args.path == "auto" else None),
            "kernel_ms": round(kernel_ms, 4),
        },
    }
    if args.op == "fwd" and not args.no_yardstick:
        # what the matrix cores sustain on this machine, same element type, N(0,1) operands in
        # registers: the published peak assumes 2.4 GHz, which the chip does not hold under load
        sustained = mfma_yardstick(w.dtype)
        result["roofline"]["mfma_sustained_tflops"] = round(sustained, 1)
        result["roofline"]["frac_of_sustained"] = round(achieved_tflops / sustained, 4)
    if not args.no_cpu_baseline:
        if args.op == "fwd" or comparison:
            rec, err = cpu_baseline(w, i32, k32, out)
        else:
            rec, err = cpu_baseline_bwd(w, args.op, i32, k32, g32, out)
        result["cpu_baseline"] = rec
        result["config"]["max_err_vs_oracle_sample"] = err
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
