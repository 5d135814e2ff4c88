#!/usr/bin/env python3
"""Benchmark of the CAT-loss hot path (forward + backward) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2_llama1b_bf16]

A step is one pass of the whole hot path over one batch of synthetic input already
resident in HBM: pard2_cat_fwd (head contraction, online log-softmax, confidence, CAT
weight, loss) followed by pard2_cat_bwd (dZ recompute, dH, dW).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 matrix-core peak

# HBM-side bytes per launch (fetch, write) from the two rocprofv3 --pmc passes summarised in
# profiles/c2_llama1b_hbm_traffic.md (FETCH_SIZE scaled by 2.0, WRITE_SIZE by 1.0 after the copy
# calibration described there).  Counters cannot be read from inside this process: the figures
# are those of the committed profile and apply to the headline workload only.
MIB = float(1 << 20)
MEASURED_TRAFFIC = {
    "c2_llama1b_bf16": {
        "fwd_stats_kernel": (6215.2 * MIB, 2.3 * MIB),
        "dz_kernel": (835.0 * MIB, 250.5 * MIB),
        "dh_kernel": (808.0 * MIB, 69.8 * MIB),
        "dw_kernel": (821.2 * MIB, 64.2 * MIB),
        # variant kd, teacher width 4096 (profiles/c2_llama1b_kd_teacher4096_kernel_trace.md)
        "kd_stats_kernel": (34700.4 * MIB, 4.4 * MIB),
        "kd_dz_kernel": (3830.4 * MIB, 250.5 * MIB),
    },
}


def make_inputs(wl, device):
    """Synthetic H, W of the workload's shape, drawn on the device; targets follow the
    workload's agreement recipe with the argmax taken from a stats-only pass of the HIP
    forward (the benchmark never calls the oracle for its inputs)."""
    import torch
    from paper_2605_08632_amd import binding as b, synth
    g = torch.Generator(device=device)
    g.manual_seed(wl.seed)
    H = torch.randn(wl.T, wl.d, generator=g, device=device, dtype=torch.float32)
    H = H / H.pow(2).mean(dim=1, keepdim=True).sqrt()
    W = torch.randn(wl.V, wl.d, generator=g, device=device, dtype=torch.float32) * (4.0 / np.sqrt(wl.d))
    H, W = H.to(torch.bfloat16), W.to(torch.bfloat16)
    desc = b.make_desc(wl.T, wl.d, wl.V, wl.B, wl.K, b.PARD2_BF16, beta=wl.beta)
    y0 = torch.zeros(wl.T, dtype=torch.int32, device=device)
    st = b.pard2_cat_fwd(desc, H, W, y0, stats_only=True)
    argmax = st["argmax"].cpu().numpy()
    y, _ = synth.make_targets(wl.seed, argmax, wl.B, wl.K, wl.V, wl.p_agree, wl.fallback)
    vl = None
    if wl.ragged_frac > 0:
        vl_np = synth.make_valid_len(wl.seed, wl.B, wl.K, wl.ragged_frac)
        y = synth.apply_tail_padding(y, vl_np, wl.K)
        vl = torch.from_numpy(vl_np).to(device)
    return desc, H, W, torch.from_numpy(y).to(device), vl


def cpu_baseline(wl, H, W, y, n_blocks):
    """The fp64 oracle, as it stands, on the first n_blocks draft blocks (all V, all d)."""
    from oracle import cat_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    Ts = n_blocks * wl.K
    Hs = H[:Ts].float().cpu().numpy()
    Wf = W.float().cpu().numpy()
    ys = y[:Ts].cpu().numpy()
    t0 = time.perf_counter()
    O.cat_loss_and_grads(Hs, Wf, ys, n_blocks, wl.K, beta=wl.beta)
    dt = time.perf_counter() - t0
    return {"value": Ts / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"fp64 numpy oracle fwd+bwd on the first {n_blocks} blocks ({Ts} of {wl.T} token rows), "
                      f"full V={wl.V}, d={wl.d}; {dt:.1f} s"}


def out_stats_argmax(b, desc, H, W, y):
    """Greedy predictions of the head (stats-only forward of the HIP path)."""
    return b.pard2_cat_fwd(desc, H, W, y, stats_only=True)["argmax"]


def measured_context(wl, H, W):
    """Context for the roofline fraction, measured on the same device (not part of the timed path):
    what the matrix cores sustain with register-resident operands (constant and random data), and
    what the vendor GEMM library reaches on the forward-shaped contraction with the same H, W."""
    import subprocess
    import torch
    ctx = {}
    tool = os.path.join(ROOT, "paper_2605_08632_amd", "mfma_peak")
    if os.path.exists(tool):
        r = subprocess.run([tool, "200"], capture_output=True, text=True, timeout=120)
        for line in r.stdout.splitlines():
            if "TFLOP/s" in line:
                key = "mfma_only_random_tflops" if line.startswith("random") else "mfma_only_constant_tflops"
                ctx[key] = float(line.split("ms")[1].split("TFLOP/s")[0])
    Hs = H[:min(wl.T, 8192)]
    for _ in range(3):
        Z = Hs @ W.t()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        Z = Hs @ W.t()
    e1.record()
    torch.cuda.synchronize()
    del Z
    ms = e0.elapsed_time(e1) / 10
    ctx["vendor_gemm_fwd_shape_tflops"] = 2.0 * Hs.shape[0] * wl.V * wl.d / (ms * 1e-3) / 1e12
    ctx["note"] = ("vendor_gemm = torch.matmul (hipBLASLt) H @ W^T materialising the logits; "
                   "mfma_only = register-resident MFMA loop, no memory traffic")
    return ctx


def bench_inject(args, wl, dev):
    """e' = e + xi Proj([l; m; h]) forward + backward (dT, dP) at the workload's T and d."""
    import torch
    from paper_2605_08632_amd import binding as b
    T, d, dt, F = wl.T, wl.d, args.teacher_d, 3
    g = torch.Generator(device=dev)
    g.manual_seed(wl.seed + 13)
    mk = lambda *shape: torch.randn(*shape, generator=g, device=dev, dtype=torch.float32)
    E = mk(T, d).to(torch.bfloat16)
    feats = [mk(T, dt).to(torch.bfloat16) for _ in range(F)]
    P = (mk(d, F * dt) / np.sqrt(F * dt)).to(torch.bfloat16)
    G = mk(T, d).to(torch.bfloat16)
    rows_per_instance = wl.K * 64
    xi = (torch.rand(T // rows_per_instance + 1, generator=g, device=dev) >= 0.1).float()
    xi = xi.repeat_interleave(rows_per_instance)[:T].contiguous()      # rho = 0.1, one draw per instance
    Eout = torch.empty_like(E)
    dP = torch.empty(d, F * dt, dtype=torch.bfloat16, device=dev)

    def step():
        b.pard2_inject_fwd(E, feats, P, xi, Eout=Eout)
        b.pard2_inject_bwd(G, feats, xi, dP=dP)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    b.pard2_cat_kernel_timing(True)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    names = ("inject_fwd_kernel", "inject_dp_kernel")
    per_kernel = {n: b.pard2_cat_kernel_timing_read(b.KERNEL_NAMES.index(n)) for n in names}
    b.pard2_cat_kernel_timing(False)
    flop = 2.0 * T * d * F * dt                      # per kernel launch (forward; dP the same)
    k = max(names, key=lambda n: per_kernel[n][0])
    k_ms, k_n = per_kernel[k]
    achieved = flop / (k_ms / k_n * 1e-3) / 1e12
    print(json.dumps({
        "metric": "gated target-feature injection fwd+bwd tokens/s (adjacent step; not the CAT-loss metric)",
        "value": T / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{wl.name} shape: T={T}, d={d}, {F} target features of width {dt}, rho=0.1, fwd+bwd"},
        "executed_tflops": 2 * flop / (ms * 1e-3) / 1e12,
        "kernel_ms_per_step": {n: per_kernel[n][0] / args.steps for n in names},
        "roofline": {"bound": "mfma", "kernel": k, "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "avg_launch_ms": k_ms / k_n,
                     "launches": k_n, "flop_per_launch": flop, "traffic": None},
    }))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--context", action="store_true",
                    help="also measure the MFMA-only peak and the vendor GEMM on this device (adds ~5 s)")
    ap.add_argument("--variant", default="cat",
                    help="cat (default) | decay0.8 | uniform | external | accumulate | fwd | stats | "
                         "kd (the Eq.12 token loss: beta CE + KD against a teacher head of width --teacher-d) | "
                         "kd-deferred (same, loss and KL returned by the backward) | "
                         "inject (gated injection of 3 target features of width --teacher-d into the draft's input "
                         "embeddings, fwd+bwd: an adjacent step, not the loss)")
    ap.add_argument("--teacher-d", type=int, default=4096, help="hidden width of the teacher head (variant kd)")
    ap.add_argument("--graph", action="store_true",
                    help="replay the step from a captured HIP graph (launch gaps removed); the per-kernel event "
                         "timing is then taken from an eager pass of the same steps run just before")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2_llama1b_bf16")
    ap.add_argument("--cpu-blocks", type=int, default=384, help="draft blocks in the oracle timing sample (0 = skip)")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="after the timed region, run one plain device copy of this many MiB (a kernel of known "
                         "HBM traffic for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
                 "(the path would shard by draft blocks, with one all-reduce of two scalars and the usual dW reduction)")

    import torch
    from paper_2605_08632_amd import binding as b, synth
    wl = synth.WORKLOADS[args.workload]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.variant == "inject":
        return bench_inject(args, wl, dev)
    desc, H, W, y, vl = make_inputs(wl, dev)
    ws = b.alloc_workspace(desc, dev)
    out = {}
    # gradient outputs rotate between two buffers from step to step (caches are not flushed otherwise)
    dHs = [torch.empty(wl.T, wl.d, dtype=torch.bfloat16, device=dev) for _ in range(2)]
    dWs = [torch.empty(wl.V, wl.d, dtype=torch.bfloat16, device=dev) for _ in range(2)]
    turn = [0]

    # comparators and partial passes (the default, "cat", is the headline path)
    conf_in, accumulate, passes = None, False, "fwd+bwd"
    if args.variant == "decay0.8":           # fixed position decay gamma^k (the ablation's comparator)
        desc.weight_mode, desc.gamma = b.PARD2_W_DECAY, 0.8
    elif args.variant == "uniform":          # plain PARD cross-entropy (Eq.5)
        desc.weight_mode = b.PARD2_W_UNIFORM
    elif args.variant == "external":         # teacher confidences supplied (the paper-exact path)
        agree = (out_stats_argmax(b, desc, H, W, y) == y).cpu().numpy()
        conf_in = torch.from_numpy(synth.make_external_conf(wl.seed, agree)).to(dev)
    elif args.variant == "accumulate":       # dW += (gradient accumulation)
        accumulate = True
        for t in dWs:
            t.zero_()
    elif args.variant == "fwd":
        passes = "fwd"
    elif args.variant == "stats":            # stats-only forward = the teacher-confidence producer
        passes = "stats"
    elif args.variant in ("kd", "kd-deferred"):   # weighted beta CE + KL(teacher || draft), two-head kernels
        # teacher recipe of synth.make_teacher, drawn on the device: draft operands extended by
        # independent columns, so that teacher logits = draft logits + noise of std ~2
        dt = args.teacher_d
        if dt <= wl.d or dt % 8:
            sys.exit("--teacher-d must exceed the draft width and be a multiple of 8")
        g = torch.Generator(device=dev)
        g.manual_seed(wl.seed + 12)
        E = torch.randn(wl.T, dt - wl.d, generator=g, device=dev, dtype=torch.float32)
        E = 2.0 * E / E.pow(2).mean(dim=1, keepdim=True).sqrt()
        Ht = torch.cat([H, E.to(torch.bfloat16)], dim=1).contiguous()
        del E
        Wt = torch.empty(wl.V, dt, dtype=torch.bfloat16, device=dev)
        Wt[:, :wl.d] = W
        Wt[:, wl.d:] = (torch.randn(wl.V, dt - wl.d, generator=g, device=dev, dtype=torch.float32)
                        / np.sqrt(dt - wl.d)).to(torch.bfloat16)
        ws = b.alloc_kd_workspace(desc, dt, dev)
    elif args.variant != "cat":
        sys.exit(f"unknown variant {args.variant}")
    kd = args.variant in ("kd", "kd-deferred")
    deferred = args.variant == "kd-deferred"   # forward without the cross term; KL and loss from the backward
    kd_late = torch.empty(wl.T, dtype=torch.float32, device=dev)
    loss_late = torch.empty(1, dtype=torch.float32, device=dev)

    def step_kd():
        turn[0] ^= 1
        dH, dW = dHs[turn[0]], dWs[turn[0]]
        o = b.pard2_cat_kd_fwd(desc, H, W, Ht, Wt, y, valid_len=vl, workspace=ws, out=out, defer_loss=deferred)
        if deferred:
            b.pard2_cat_kd_bwd(desc, H, W, Ht, Wt, y, o["lse"], o["lse_t"], o["w"], valid_len=vl, dH=dH, dW=dW,
                               workspace=ws, logp_y=o["logp_y"], kd=kd_late, loss=loss_late)
        else:
            b.pard2_cat_kd_bwd(desc, H, W, Ht, Wt, y, o["lse"], o["lse_t"], o["w"], valid_len=vl, dH=dH, dW=dW,
                               workspace=ws)

    def step():
        if kd:
            return step_kd()
        turn[0] ^= 1
        dH, dW = dHs[turn[0]], dWs[turn[0]]
        o = b.pard2_cat_fwd(desc, H, W, y, conf_in=conf_in, valid_len=vl, workspace=ws, out=out,
                            stats_only=(passes == "stats"))
        if passes == "fwd+bwd":
            b.pard2_cat_bwd(desc, H, W, y, o["lse"], o["w"], valid_len=vl, dH=dH, dW=dW, workspace=ws,
                            accumulate_dW=accumulate)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    b.pard2_cat_kernel_timing(True)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    per_kernel = [b.pard2_cat_kernel_timing_read(k) for k in range(len(b.KERNEL_NAMES))]
    b.pard2_cat_kernel_timing(False)
    if args.graph:                              # same K steps again, as one graph replay per step
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            graph.replay()
        e1.record()
        torch.cuda.synchronize()
        ms_eager, ms = ms, e0.elapsed_time(e1) / args.steps

    if args.calib_copy_mib > 0:
        src = torch.empty(args.calib_copy_mib << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                       # reads and writes calib_copy_mib MiB each
        torch.cuda.synchronize()
        del src, dst

    n_valid = int((y >= 0).sum().item())
    bwd = passes == "fwd+bwd"
    flops_model = (6.0 if bwd else 2.0) * n_valid * wl.V * wl.d
    flops_exec = (8.0 if bwd else 2.0) * wl.T * wl.V * wl.d
    if kd:                                   # + the teacher head: once in the loss, once more in the recompute
        flops_model += 2.0 * n_valid * wl.V * args.teacher_d
        flops_exec += 4.0 * wl.T * wl.V * args.teacher_d
    if not bwd:
        n_valid = wl.T                       # a forward sweep produces statistics for every row
    # dominant kernel = largest share of the step; per step each single-head kernel runs 2*T*V*d flops in
    # total, each two-head kernel 2*T*V*(d + dt)
    tot = [p[0] for p in per_kernel]
    k = int(np.argmax(tot))
    k_ms, k_n = per_kernel[k]
    width = wl.d + args.teacher_d if b.KERNEL_NAMES[k].startswith("kd_") else wl.d
    flops_kernel_per_launch = 2.0 * wl.T * wl.V * width * args.steps / max(k_n, 1)
    achieved = flops_kernel_per_launch / (k_ms / max(k_n, 1) * 1e-3) / 1e12
    tr = MEASURED_TRAFFIC.get(wl.name, {}).get(b.KERNEL_NAMES[k])
    if b.KERNEL_NAMES[k].startswith("kd_") and args.teacher_d != 4096:
        tr = None                                # the stored counters are for the 4096-wide teacher
    traffic = None if tr is None else tr[0] + tr[1]           # bytes per launch
    traffic_detail = None if tr is None else {"fetch_bytes": tr[0], "write_bytes": tr[1],
                                              "source": "profiles/c2_llama1b_kd_teacher4096_kernel_trace.md"
                                              if b.KERNEL_NAMES[k].startswith("kd_") else
                                              "profiles/c2_llama1b_hbm_traffic.md"}
    res = {
        "metric": "CAT loss fwd+bwd tokens/s and % bf16 MFMA peak, d=2048 V=128256 T=8192",
        "value": n_valid / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: T={wl.T} ({wl.B} blocks x K={wl.K}), d={wl.d}, V={wl.V}, "
                               f"variant {args.variant}{f' (teacher d={args.teacher_d})' if kd else ''}, beta={wl.beta}, {passes}"},
        "model_tflops": flops_model / (ms * 1e-3) / 1e12,
        "pct_bf16_mfma_peak_model_flops": 100.0 * flops_model / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "executed_tflops": flops_exec / (ms * 1e-3) / 1e12,
        "kernel_ms_per_step": {b.KERNEL_NAMES[i]: per_kernel[i][0] / args.steps
                               for i in range(len(b.KERNEL_NAMES)) if per_kernel[i][1] > 0},
        "roofline": {"bound": "mfma", "kernel": b.KERNEL_NAMES[k], "achieved": achieved,
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                     "avg_launch_ms": k_ms / max(k_n, 1), "launches": k_n,
                     "flop_per_launch": flops_kernel_per_launch, "traffic": traffic,
                     "traffic_detail": traffic_detail},
    }
    if args.graph:
        res["config"]["launch"] = "HIP graph replay"
        res["ms_per_step_eager"] = ms_eager
    if args.context:
        res["context"] = measured_context(wl, H, W)
    if args.cpu_blocks > 0 and args.variant == "cat":
        res["cpu_baseline"] = cpu_baseline(wl, H, W, y, min(args.cpu_blocks, wl.B))
    print(json.dumps(res))


if __name__ == "__main__":
    main()
