#!/usr/bin/env python3
"""Throughput of the conv1d sub-block hot path on one MI355X.

A step is one pass of the whole hot path over one synthetic batch of the headline workload
(Jasper B3-shaped block: B=32, Cin=Cout=512, T=800, K=17, stride 1, pad 8, bf16 storage,
float32 accumulation, folded-BN affine + residual + ReLU):
    nm_conv1d_block_fwd  ->  nm_conv1d_bwd_data (dx and dres)  ->  nm_conv1d_bwd_weight
with every helper kernel of those calls (weight packing, dz pass, dw reduction) inside the timed
region and all inputs resident in HBM before it starts.  The same step with both gradients from one
call (nm_conv1d_bwd) is timed afterwards and reported as an extra object, not as the headline.  The metric is
3 * 2*B*Cout*T_out*Cin*K flop per step divided by the measured time, in TFLOP/s.

The JSON line also carries
  roofline     -- the dominant kernel (largest share of the step) against the bf16 dense MFMA
                  peak; its average duration is measured in the timed region with HIP events
                  recorded on the launch stream right around that kernel (the library's
                  nm_conv1d_time_next_main_kernel hook) in every fourth step;
  cpu_baseline -- the fp64 CPU oracle, untuned, timed on the host cores on the first 8 of the
                  32 batch items of the same workload (a baseline, not the target).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak (published)


def cpu_baseline(cfg_full):
    """Oracle forward + both gradients on a bounded sample (first 8 batch items)."""
    import numpy as np
    import _util as U
    from oracle import conv1d_oracle as orc
    from paper_1909_09577_amd import inputs as syn
    nb = min(8, cfg_full.B)
    cfg = syn.shrink(cfg_full, B=nb)
    inp = syn.make_inputs(cfg, "bf16")
    t0 = time.perf_counter()
    y = U.oracle_fwd(cfg, inp)
    dx, dw, dres = U.oracle_bwd(cfg, inp, y)
    dt = time.perf_counter() - t0
    flops = 3 * cfg.flops_per_pass
    return {"value": round(flops / dt / 1e12, 6), "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"first {nb} of {cfg_full.B} batch items of the same workload, fp64, fwd+dgrad+wgrad, {dt:.1f} s"}


def recorded_traffic(kernel_key):
    """HBM bytes per launch of a kernel from profiles/hbm_traffic_b3_512_k17.md, or None when that
    file is missing or the kernel sources have changed since the counters were taken."""
    import hashlib
    import re
    path = os.path.join(ROOT, "profiles", "hbm_traffic_b3_512_k17.md")
    if not os.path.exists(path):
        return None
    text = open(path).read()
    m = re.search(r"sources_sha256:\s*([0-9a-f]{64})", text)
    if not m:
        return None
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_1909_09577_amd", "csrc")
    for f in sorted(os.listdir(csrc)):
        if f.endswith((".hip", ".h")):
            h.update(open(os.path.join(csrc, f), "rb").read())
    if h.hexdigest() != m.group(1):
        return None
    m = re.search(r"^\|\s*%s\s*\|.*\|\s*([0-9.]+)\s*MB\s*\|\s*$" % re.escape(kernel_key), text, re.M)
    return float(m.group(1)) * 1e6 if m else None


def stack_report():
    """Time of one forward+backward step of the whole 64-layer 10x5-shaped stack (B=32, T=1600->800):
    every distinct layer shape is timed on its own (block forward + nm_conv1d_bwd) and weighted with
    the number of times it occurs; prints one JSON line.  Not the headline: `--stack` only."""
    import torch
    from paper_1909_09577_amd import binding as nm
    from paper_1909_09577_amd import inputs as syn
    groups = {}
    for e in syn.jasper_10x5_layers():
        c = e["cfg"]
        key = (c.Cin, c.Cout, c.K, c.stride, c.dilation, c.residual, c.affine, c.relu, c.T)
        groups.setdefault(key, [0, c])[0] += 1
    total_ms = total_flop = 0.0
    rows = []
    for cnt, c in groups.values():
        To = c.T_out
        x = torch.randn(c.B, c.Cin, c.T, device="cuda").bfloat16()
        w = (torch.randn(c.Cout, c.Cin, c.K, device="cuda") / (c.Cin * c.K) ** 0.5).bfloat16()
        dy = torch.randn(c.B, c.Cout, To, device="cuda").bfloat16()
        res = torch.randn(c.B, c.Cout, To, device="cuda").bfloat16() if c.residual else None
        scale = (torch.rand(c.Cout, device="cuda") + 0.5) if c.affine else None
        shift = torch.randn(c.Cout, device="cuda") * 0.1 if c.affine else None
        y = torch.empty(c.B, c.Cout, To, device="cuda", dtype=torch.bfloat16)
        dx = torch.empty_like(x)
        dres = torch.empty_like(y) if c.residual else None
        dw = torch.empty(c.Cout, c.Cin, c.K, device="cuda")
        kw = dict(stride=c.stride, dilation=c.dilation, pad=c.pad)
        ws = torch.empty(max(nm.nm_conv1d_workspace_bytes(op, *c.dims(), nm.NM_BF16, nm.NM_RELU) for op in (0, 3)) + 256,
                         dtype=torch.uint8, device="cuda")

        def step():
            nm.nm_conv1d_block_fwd(x, w, scale, shift, res, y=y, relu=c.relu, workspace=ws, **kw)
            nm.nm_conv1d_bwd(x, dy, w, y=y if c.relu else None, scale=scale, dx=dx, dres=dres, dw=dw, relu=c.relu,
                             workspace=ws, **kw)

        for _ in range(3):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        n = 10
        for _ in range(n):
            step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / n * 1e3
        total_ms += ms * cnt
        total_flop += 3 * c.flops_per_pass * cnt
        rows.append({"layer": f"{c.Cin}->{c.Cout} K={c.K} s={c.stride} d={c.dilation}" + (" +res" if c.residual else ""),
                     "count": cnt, "ms": round(ms, 4), "TFLOP/s": round(3 * c.flops_per_pass / ms / 1e9, 1)})
    print(json.dumps({"metric": "10x5 stack fwd+bwd, layer by layer (bf16)", "ms_per_step": round(total_ms, 3),
                      "value": round(total_flop / total_ms / 1e9, 1), "unit": "TFLOP/s",
                      "frac_of_bf16_mfma_peak": round(total_flop / total_ms / 1e9 / PEAK_BF16_TFLOPS, 4),
                      "layers": sorted(rows, key=lambda r: -r["ms"] * r["count"])}), flush=True)


def decoder_report(steps, warmup, with_cpu):
    """Decoder tail (1x1 convolution to 29 classes + log-softmax) at the encoder's output size; an
    HBM-bound step: one JSON line with the achieved bandwidth on its algorithmic bytes.  `--decoder` only."""
    import numpy as np
    import torch
    from paper_1909_09577_amd import binding as nm
    B, Cin, Ncls, T = 32, 1024, 29, 800
    x = torch.randn(B, Cin, T, device="cuda").bfloat16()
    w = (torch.randn(Ncls, Cin, device="cuda") / Cin ** 0.5).bfloat16()
    bias = torch.randn(Ncls, device="cuda") * 0.5
    logp = torch.empty(B, Ncls, T, device="cuda")
    for _ in range(max(warmup, 1)):
        nm.nm_decoder_logsoftmax_fwd(x, w, bias, logp)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()  # the kernel runs on torch's current stream, the one these events are recorded on
    for _ in range(steps):
        nm.nm_decoder_logsoftmax_fwd(x, w, bias, logp)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    nbytes = x.numel() * 2 + w.numel() * 2 + bias.numel() * 4 + logp.numel() * 4
    gbs = nbytes / (ms * 1e-3) / 1e9
    out = {"metric": "decoder tail: 1x1 conv 1024->29 + log-softmax, frames/s", "value": round(B * T / (ms * 1e-3), 1),
           "unit": "frames/s", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms, 5),
           "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": "B=32 Cin=1024 Ncls=29 T=800"},
           "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": 8000.0, "unit": "GB/s",
                        "frac": round(gbs / 8000.0, 4), "traffic": None, "kernel": "decoder_mfma_kernel",
                        "bytes_per_launch": nbytes}}
    if with_cpu:
        from oracle import decoder_oracle as dorc
        nb = 8
        xs, ws, bs = x[:nb].float().cpu().numpy(), w.float().cpu().numpy(), bias.cpu().numpy()
        t0 = time.perf_counter()
        dorc.decoder_logsoftmax(xs, ws, bs)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(nb * T / dt, 1), "unit": "frames/s", "cores": os.cpu_count(), "kind": "oracle",
                               "sample": f"first {nb} of {B} batch items, float64 numpy, {dt:.2f} s"}
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--calibration-copies", type=int, default=0,
                    help="run this many plain 256 MiB copy kernels (dst = src + 1) before the steps (counter runs only: "
                         "the copy kernel's FETCH_SIZE / WRITE_SIZE per byte moved scale the other kernels' counters)")
    ap.add_argument("--stack", action="store_true",
                    help="instead of the headline: time every layer shape of the 64-layer stack (one extra JSON line)")
    ap.add_argument("--decoder", action="store_true",
                    help="instead of the headline: the decoder tail (1x1 conv + log-softmax), an HBM-bound step")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    import _util as U
    from paper_1909_09577_amd import binding as nm
    from paper_1909_09577_amd import inputs as syn

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    nm.lib()  # fails loudly if the HIP library has not been built
    if args.stack:
        stack_report()
        return
    if args.decoder:
        decoder_report(args.steps, args.warmup, not args.no_cpu_baseline)
        return

    cfg = syn.HEADLINE
    dt = "bf16"
    inp = syn.make_inputs(cfg, dt)
    kw = U.geom_kw(cfg)
    x, w = U.to_dev(inp, "x", dt), U.to_dev(inp, "w", dt)
    scale, shift = U.to_dev(inp, "scale", dt), U.to_dev(inp, "shift", dt)
    res, dy = U.to_dev(inp, "residual", dt), U.to_dev(inp, "dy", dt)
    To = cfg.T_out
    y = torch.empty((cfg.B, cfg.Cout, To), dtype=torch.bfloat16, device="cuda")
    dx = torch.empty_like(x)
    dres = torch.empty_like(y)
    dw = torch.empty((cfg.Cout, cfg.Cin, cfg.K), dtype=torch.float32, device="cuda")
    ws_bytes = max(nm.nm_conv1d_workspace_bytes(op, *cfg.dims(), nm.NM_BF16, nm.NM_RELU) for op in (0, 1, 2))
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device="cuda")

    def ev():
        e = torch.cuda.Event(enable_timing=True)
        e.record()  # torch creates the handle on first record
        return e

    names = ("fwd", "dgrad", "wgrad")
    # Events around a kernel split the stream's back-to-back dispatch (a few microseconds per pair), so
    # the timed region carries them only around the dominant kernel and only in every fourth step; which
    # kernel dominates is found with events around all three during the warmup steps.
    every = 4
    warm_pairs = {n: [(ev(), ev()) for _ in range(max(args.warmup, 1))] for n in names}
    timed_steps = list(range(0, args.steps, every))
    pairs = [(ev(), ev()) for _ in timed_steps]

    def step(hook=None):
        if hook and "fwd" in hook:
            nm.nm_conv1d_time_next_main_kernel(*hook["fwd"])
        nm.nm_conv1d_block_fwd(x, w, scale, shift, res, y=y, relu=True, workspace=ws, **kw)
        if hook and "dgrad" in hook:
            nm.nm_conv1d_time_next_main_kernel(*hook["dgrad"])
        nm.nm_conv1d_bwd_data(dy, w, cfg.T, y=y, scale=scale, dx=dx, dres=dres, relu=True, workspace=ws, **kw)
        if hook and "wgrad" in hook:
            nm.nm_conv1d_time_next_main_kernel(*hook["wgrad"])
        nm.nm_conv1d_bwd_weight(x, dy, cfg.K, y=y, scale=scale, dw=dw, relu=True, workspace=ws, **kw)

    if args.calibration_copies:
        # an elementwise kernel that reads 256 MiB and writes 256 MiB (a device-to-device memcpy may go
        # through a DMA engine and never show up as a kernel)
        src = torch.arange(64 << 20, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(args.calibration_copies):
            torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst

    for i in range(max(args.warmup, 1)):
        step({n: warm_pairs[n][i] for n in names})
    torch.cuda.synchronize()
    warm_ms = {n: sorted(a.elapsed_time(b) for a, b in warm_pairs[n])[len(warm_pairs[n]) // 2] for n in names}
    dominant = max(warm_ms, key=warm_ms.get)

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step({dominant: pairs[i // every]} if i % every == 0 else None)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    # the same step with both gradients from one call (nm_conv1d_bwd): reported beside the headline
    ws_f = torch.empty(max(nm.nm_conv1d_workspace_bytes(nm.NM_OP_BWD, *cfg.dims(), nm.NM_BF16, nm.NM_RELU), 256),
                       dtype=torch.uint8, device="cuda")

    def step_fused():
        nm.nm_conv1d_block_fwd(x, w, scale, shift, res, y=y, relu=True, workspace=ws, **kw)
        nm.nm_conv1d_bwd(x, dy, w, y=y, scale=scale, dx=dx, dres=dres, dw=dw, relu=True, workspace=ws_f, **kw)

    for _ in range(max(args.warmup, 1)):
        step_fused()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        step_fused()
    torch.cuda.synchronize()
    ms_fused = (time.perf_counter() - t1) / args.steps * 1e3

    # per-pass times (event pairs around each call, helper kernels included) and a cold variant of the
    # step: six buffer sets (about 1 GB, four times the 256 MB Infinity Cache) used in rotation, so that
    # no tensor is found in a cache from the previous step.  Reported beside the headline, which is the
    # warm step above (the tensors of one layer stay resident between its forward and backward pass).
    def timed(fn, n):
        a, b = ev(), ev()
        a.record()
        for _ in range(n):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    n_pass = max(args.steps // 4, 10)
    per_pass = {
        "fwd": timed(lambda: nm.nm_conv1d_block_fwd(x, w, scale, shift, res, y=y, relu=True, workspace=ws, **kw), n_pass),
        "dgrad": timed(lambda: nm.nm_conv1d_bwd_data(dy, w, cfg.T, y=y, scale=scale, dx=dx, dres=dres, relu=True,
                                                     workspace=ws, **kw), n_pass),
        "wgrad": timed(lambda: nm.nm_conv1d_bwd_weight(x, dy, cfg.K, y=y, scale=scale, dw=dw, relu=True, workspace=ws,
                                                       **kw), n_pass),
    }
    sets = [tuple(torch.empty_like(t).copy_(t) for t in (x, res, dy, y, dx, dres)) for _ in range(6)]
    state = {"i": 0}

    def cold_step():
        xs, rs, dys, ys, dxs, drs = sets[state["i"] % len(sets)]
        state["i"] += 1
        nm.nm_conv1d_block_fwd(xs, w, scale, shift, rs, y=ys, relu=True, workspace=ws, **kw)
        nm.nm_conv1d_bwd_data(dys, w, cfg.T, y=ys, scale=scale, dx=dxs, dres=drs, relu=True, workspace=ws, **kw)
        nm.nm_conv1d_bwd_weight(xs, dys, cfg.K, y=ys, scale=scale, dw=dw, relu=True, workspace=ws, **kw)

    for _ in range(len(sets)):
        cold_step()
    ms_cold = timed(cold_step, max(args.steps // 4, 12))
    del sets

    ms_per_step = elapsed / args.steps * 1e3
    flops_step = 3 * cfg.flops_per_pass
    value = flops_step / (ms_per_step * 1e-3) / 1e12

    dom_ms = sum(a.elapsed_time(b) for a, b in pairs) / len(pairs)
    kernel_names = {"fwd": "conv_gemm_kernel<5,1,17> (forward)", "dgrad": "conv_gemm_kernel<5,1,17> (input gradient)",
                    "wgrad": "wgrad_shared_kernel<17, 1>"}
    achieved = cfg.flops_per_pass / (dom_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "achieved": round(achieved, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": recorded_traffic(dominant),
                "kernel": kernel_names[dominant],
                "flops_per_launch": cfg.flops_per_pass,
                "avg_launch_ms": round(dom_ms, 4), "timed_launches": len(pairs),
                "warmup_main_kernels_ms": {n: round(v, 4) for n, v in warm_ms.items()}}

    out = {
        "metric": "conv1d fwd+dgrad+wgrad TFLOP/s (bf16), C=512 K=17 T=800",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "Jasper B3-shaped block: B=32 Cin=Cout=512 T=800 K=17 stride 1 dilation 1 pad 8, "
                               "affine+residual+ReLU, fwd+dgrad(+dres)+wgrad", "seed": cfg.seed},
        "frac_of_bf16_mfma_peak": round(value / PEAK_BF16_TFLOPS, 4),
        "per_pass_ms": {n: round(v, 4) for n, v in per_pass.items()},
        "per_pass_tflops": {n: round(cfg.flops_per_pass / (v * 1e-3) / 1e12, 1) for n, v in per_pass.items()},
        "cold": {"ms_per_step": round(ms_cold, 4), "value": round(flops_step / (ms_cold * 1e-3) / 1e12, 2), "unit": "TFLOP/s",
                 "note": "six rotating sets of activation tensors (about 1 GB), nothing cached from the previous step"},
        "fused_backward": {"ms_per_step": round(ms_fused, 4), "value": round(flops_step / (ms_fused * 1e-3) / 1e12, 2),
                           "unit": "TFLOP/s", "note": "same step with nm_conv1d_bwd (one dz pass for both gradients)"},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
