#!/usr/bin/env python3
"""Benchmark of the dilated flash attention forward on one MI355X.

A step is one pass of the whole hot path (gather + attention + placement + branch merge,
one dfa_forward call) over one synthetic batch of the throughput workload: B = 16 images of
64x64 = 4096 tokens, 12 heads x 64, bf16, branches (1024,1), (2048,2), (4096,4).
Prints ONE JSON line.  Inputs are resident in HBM before the timed region starts.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16 matrix peak (published)
WORKLOAD = "throughput"
# HBM bytes per launch, from the counter runs: rocprofv3 FETCH_SIZE and WRITE_SIZE per dispatch, scaled by what the
# same counters read for a plain copy of known size.  `bench.py --write-traffic <dir>` writes this file from
# the four counter runs; the default line reads it (null when the workload has no entry).
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "dfa_fwd_hbm_traffic.txt")
# Launches back to back before anything is timed.  At the start of a burst of launches the chip runs the
# first four or so at full speed, then drops its clock for some twenty launches and comes back to a steady
# value after about a hundred (30 ms); any idle gap of a few milliseconds starts this over (per-launch HIP-event
# times, profiles/dfa_fwd_bf16_throughput.md).  The workload asks for steady-state throughput, so every timed
# region is preceded by this many milliseconds of untimed launches; the line says how many that was.
SETTLE_MS = 150.0


HBM_PEAK_GBS = 8000.0               # MI355X HBM3E (published)


def settle(torch, fn, ms=SETTLE_MS):
    """Runs fn back to back for about `ms` milliseconds (at least 20 calls), untimed; returns the number of calls."""
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(5):
        fn()
    torch.cuda.synchronize()
    per_call = max((time.perf_counter() - t0) / 5, 1e-6)
    n = int(min(max(ms * 1e-3 / per_call, 20), 20000))
    for _ in range(n):
        fn()
    return n + 5


def read_traffic(workload):
    """HBM bytes per launch of `workload` from TRAFFIC_FILE (lines: workload=<name> ... traffic_bytes=<n>), or None."""
    try:
        for ln in open(TRAFFIC_FILE):
            kv = dict(tok.split("=", 1) for tok in ln.split() if "=" in tok)
            if kv.get("workload") == workload and "traffic_bytes" in kv:
                return int(kv["traffic_bytes"])
    except OSError:
        pass
    return None


def write_traffic(dirname):
    """Reads the counter runs under `dirname` (sub-folders <workload>_fetch, <workload>_write, copy_fetch,
    copy_write, each holding rocprofv3's *counter_collection.csv) and rewrites TRAFFIC_FILE."""
    import csv
    import glob

    def mean_counter(sub, counter, kernel_part):
        vals = []
        for path in glob.glob(os.path.join(dirname, sub, "**", "*counter_collection.csv"), recursive=True):
            for row in csv.DictReader(open(path)):
                if row["Counter_Name"] == counter and kernel_part in row["Kernel_Name"]:
                    vals.append(float(row["Counter_Value"]))
        if not vals:
            raise SystemExit(f"bench.py: no {counter} rows for {kernel_part} under {dirname}/{sub}")
        return sum(vals) / len(vals), len(vals)

    copy_kib = (1 << 28) / 1024.0                     # --copy-calibration copies 256 MiB each way
    f_copy, _ = mean_counter("copy_fetch", "FETCH_SIZE", "opy")
    w_copy, _ = mean_counter("copy_write", "WRITE_SIZE", "opy")
    f_fac, w_fac = copy_kib / f_copy, copy_kib / w_copy
    lines = ["# HBM traffic per launch of dfa_fwd_bf16_kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch, mean over the",
             "# dispatches of one run), scaled by what the same counters read for a 256 MiB device-to-device copy.",
             "# Written by `python3 bench.py --write-traffic <dir>`; read by bench.py for roofline.traffic.",
             f"copy_calibration FETCH_SIZE_KiB={f_copy:.0f} WRITE_SIZE_KiB={w_copy:.0f} fetch_factor={f_fac:.4f} write_factor={w_fac:.4f}"]
    for sub in sorted(os.listdir(dirname)):
        if sub.endswith("_fetch") and sub != "copy_fetch":
            wl = sub[:-len("_fetch")]
            f, nf = mean_counter(sub, "FETCH_SIZE", "dfa_fwd")
            w, nw = mean_counter(wl + "_write", "WRITE_SIZE", "dfa_fwd")
            total = int(round((f * f_fac + w * w_fac) * 1024))
            lines.append(f"workload={wl} FETCH_SIZE_KiB={f:.0f} WRITE_SIZE_KiB={w:.0f} dispatches={nf} "
                         f"read_bytes={int(f * f_fac * 1024)} written_bytes={int(w * w_fac * 1024)} traffic_bytes={total}")
    open(TRAFFIC_FILE, "w").write("\n".join(lines) + "\n")
    print("\n".join(lines))


def stage_report(binding, torch, q, k, v, branches, scale, steps, warmup):
    """Achieved HBM GB/s of the unfused stage entry points (algorithmic bytes / HIP-event time).

    Algorithmic bytes per launch: gather 2*D*esize per kept row; placement D*esize*(1 + 1/r) per
    token-head; merge nb*(4*D + 4) read + D*esize + 4 written per token-head.  The unmerged
    branch launches are reported in TFLOP/s (they are the attention kernel on one branch).
    """
    Bsz, N, H, D = q.shape
    esize = q.element_size()

    def timed(fn):
        settle(torch, fn, 60.0)
        for _ in range(warmup):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps            # ms

    rows = []
    for (w, r) in branches:
        xg = binding.gather(k, w, r)
        ms = timed(lambda: binding.gather(k, w, r, out=xg))
        nbytes = 2 * Bsz * H * (N // r) * D * esize
        rows.append({"kernel": "gather_kernel", "branch": [w, r], "ms": ms, "bytes": nbytes,
                     "GB/s": nbytes / ms / 1e6, "frac_of_hbm_peak": nbytes / ms / 1e6 / HBM_PEAK_GBS})
    for (w, r) in branches:
        og = binding.gather(k, w, r)
        placed = binding.scatter(og, N, w, r)
        ms = timed(lambda: binding.scatter(og, N, w, r, out=placed))
        nbytes = Bsz * N * H * D * esize + Bsz * H * (N // r) * D * esize
        rows.append({"kernel": "scatter_kernel", "branch": [w, r], "ms": ms, "bytes": nbytes,
                     "GB/s": nbytes / ms / 1e6, "frac_of_hbm_peak": nbytes / ms / 1e6 / HBM_PEAK_GBS})
        del og
    parts = []
    for (w, r) in branches:
        ob, lb = binding.forward_branch(q, k, v, w, r, scale)
        ms = timed(lambda: binding.forward_branch(q, k, v, w, r, scale, out_b=ob, lse_b=lb))
        fl = 4 * D * Bsz * H * N * w // (r * r)
        rows.append({"kernel": "dfa_fwd_bf16_kernel<float> (one branch, unmerged)", "branch": [w, r], "ms": ms,
                     "flops": fl, "TFLOP/s": fl / ms / 1e9})
        parts.append((ob, lb))
    out_b = torch.stack([p[0] for p in parts])
    lse_b = torch.stack([p[1] for p in parts])
    del parts
    mo, ml = binding.merge(out_b, lse_b, q.dtype)
    ms = timed(lambda: binding.merge(out_b, lse_b, q.dtype, out=mo, lse=ml))
    nb = len(branches)
    nbytes = Bsz * N * H * (nb * (4 * D + 4) + D * esize + 4)
    rows.append({"kernel": "merge_kernel", "branches": nb, "ms": ms, "bytes": nbytes,
                 "GB/s": nbytes / ms / 1e6, "frac_of_hbm_peak": nbytes / ms / 1e6 / HBM_PEAK_GBS})
    unfused_ms = sum(r_["ms"] for r_ in rows if r_["kernel"].startswith("dfa_fwd")) + ms
    return {"stages": rows, "hbm_peak_GB/s": HBM_PEAK_GBS, "steps": steps, "warmup": warmup,
            "unfused_path_ms": unfused_ms,
            "note": "unfused_path_ms = the three unmerged branch launches + merge; the fused dfa_forward does all of it in one launch"}


def sweep_report(binding, synth, torch, np, steps, warmup, only=None):
    """Section 4.3's ablation (Fig. 4) as a synthetic sweep: image sizes 256^2, 512^2, 1024^2 (N = 256, 1024, 4096
    tokens of 16 x 16 patches), embed 384 (6 heads) and 768 (12 heads), B = 16.  For each shape: the three
    dilated branches scaled to it ((N/4, 1), (N/2, 2), (N, 4)) through dfa_forward; dense attention over all N
    tokens through dfa_forward (one branch with w = N, r = 1: "FlashAttention on"); and dense attention with the
    score matrix held in memory (dfa_dense_unfused: "FlashAttention off").  only = (image side, heads): that row alone
    (for a kernel trace of one shape)."""
    rows = []
    Bsz, D, scale = 16, 64, 0.125
    for H in (6, 12):
        for N in (256, 1024, 4096):
            if only and (int(N ** 0.5) * 16, H) != tuple(only):
                continue
            st, _ = synth.qkv(synth.BASE_SEED + 10 + H + N, Bsz, N, H, D, "bf16")
            q, k, v = (torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda() for a in st)
            out = torch.empty_like(q)
            lse = torch.empty((Bsz, H, N), dtype=torch.float32, device="cuda")
            dil = [(N // 4, 1), (N // 2, 2), (N, 4)]
            res = {"image": f"{int(N ** 0.5) * 16}^2", "N": N, "H": H, "B": Bsz}
            for name, br in (("dilated", dil), ("dense", [(N, 1)])):
                need = binding.workspace_bytes(Bsz, H, N, D, binding.DFA_BF16, br)
                ws = torch.empty((need,), dtype=torch.uint8, device="cuda") if need else None
                settle(torch, lambda: binding.forward(q, k, v, br, scale, out=out, lse=lse, workspace=ws), 60.0)
                ms = binding.forward_timed(q, k, v, br, scale, max(steps // 4, 10), out=out, lse=lse, workspace=ws)
                fl = synth.useful_flops(Bsz, H, N, D, br)
                res[name] = {"us": ms * 1e3, "useful_TFLOP/s": fl / ms / 1e9, "flops": fl}
            # dense attention with the scores in memory: four launches per call
            dws = torch.empty((binding.lib().dfa_dense_unfused_workspace_bytes(Bsz, H, N, D),), dtype=torch.uint8, device="cuda")
            run = lambda: binding.dense_unfused(q, k, v, scale, out=out, lse=lse, workspace=dws)
            settle(torch, run, 60.0)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            it = max(steps // 4, 10)
            e0.record()
            for _ in range(it):
                run()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / it
            fl = synth.useful_flops(Bsz, H, N, D, [(N, 1)])
            res["dense_unfused"] = {"us": ms * 1e3, "useful_TFLOP/s": fl / ms / 1e9, "flops": fl,
                                    "score_matrix_bytes": Bsz * H * N * N * 2}
            res["dense_over_dilated_time"] = res["dense"]["us"] / res["dilated"]["us"]
            res["unfused_over_fused_dense_time"] = res["dense_unfused"]["us"] / res["dense"]["us"]
            rows.append(res)
            del dws
    return {"sweep": rows, "note": "useful FLOPs = 4*D per (query, key) pair the method computes; dense attention "
                                    "computes N^2 pairs per head, the three branches 7*N^2/16; dense_unfused = scores "
                                    "materialised in memory as bf16 (QK^T product, row softmax, PV product)"}


def tile_cost_report(binding, synth, torch, np):
    """What a 64-key step and what a tile cost: single-branch launches (w, 1) on the throughput shape give
    16 * B * H tiles of w / 64 steps each; with 512 workgroup slots on the chip a launch then takes about
    c + (tiles / 512) * (per_tile + steps * per_step).  Least squares over two batch sizes and five w."""
    H, N, D, scale = 12, 4096, 64, 0.125
    rows, A, y = [], [], []
    for Bsz in (16, 32):
        st, _ = synth.qkv(synth.BASE_SEED + 40 + Bsz, Bsz, N, H, D, "bf16")
        q, k, v = (torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda() for a in st)
        out = torch.empty_like(q)
        lse = torch.empty((Bsz, H, N), dtype=torch.float32, device="cuda")
        for w in (256, 512, 1024, 2048, 4096):
            br = [(w, 1)]
            settle(torch, lambda: binding.forward(q, k, v, br, scale, out=out, lse=lse), 60.0)
            us = 1e3 * min(binding.forward_timed(q, k, v, br, scale, 30, out=out, lse=lse) for _ in range(3))
            per_slot = Bsz * H * (N // 256) / 512.0
            rows.append({"B": Bsz, "w": w, "steps_per_tile": w // 64, "tiles_per_slot": per_slot, "launch_us": us})
            A.append([1.0, per_slot, per_slot * (w // 64)])
            y.append(us)
        del q, k, v, out, lse
    coef, *_ = np.linalg.lstsq(np.array(A), np.array(y), rcond=None)
    return {"tile_cost": rows, "fit_us": {"per_launch": coef[0], "per_tile_and_slot": coef[1], "per_step_and_slot": coef[2]},
            "note": "two workgroup slots share a CU; launch_us is the best HIP-event mean of three runs of 30 launches"}


def stack_report(binding, synth, torch, np, steps, warmup, cpu_baseline, layers=12, H=12, batch=None):
    """The encoder attention stack: 12 layers, embed 768 = 12 heads x 64, B = 8 images of 4096 tokens, bf16;
    per layer QKV projection (768 -> 2304), dilated attention, output projection (768 -> 768); weights
    N(0, 0.02^2), input N(0, 1), no bias, residual or normalisation.  One step = all 12 layers."""
    cfg = synth.CONFIGS["stack_layer"]
    Bsz, N, D, branches = batch or cfg["B"], cfg["N"], cfg["D"], cfg["branches"]
    E, scale, seed = H * D, 1.0 / (D ** 0.5), cfg["seed"]

    def dev(bits):
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()

    xb, xe = synth.tensor(seed, synth.TENSOR_X, (Bsz, N, E), "bf16")
    wq_bits, wo_bits = [], []
    for l in range(layers):
        wq_bits.append(synth.tensor(seed, 10 + 2 * l, (3 * E, E), "bf16", std=0.02)[0])
        wo_bits.append(synth.tensor(seed, 11 + 2 * l, (E, E), "bf16", std=0.02)[0])
    x, wq, wo = dev(xb), dev(np.stack(wq_bits)), dev(np.stack(wo_bits))
    ws = (torch.empty((Bsz, N, 3, H, D), dtype=torch.bfloat16, device="cuda"),
          torch.empty((Bsz, N, H, D), dtype=torch.bfloat16, device="cuda"),
          torch.empty((Bsz, N, E), dtype=torch.bfloat16, device="cuda"))

    def run():
        return binding.encoder_stack(x, wq, wo, H, branches, scale, buffers=ws)

    n_settle = settle(torch, run)
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps
    M = Bsz * N
    fl_attn = synth.useful_flops(Bsz, H, N, D, branches)
    fl_qkv, fl_out = 2 * M * 3 * E * E, 2 * M * E * E
    flops = layers * (fl_attn + fl_qkv + fl_out)

    def timed(fn, it=50):
        settle(torch, fn, 60.0)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(it):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / it

    qkv, attn, y = ws
    ms_qkv = timed(lambda: binding.linear(x, wq[0], out=qkv.view(Bsz, N, 3 * E)))
    ms_attn = timed(lambda: binding.forward(qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], branches, scale, out=attn, want_lse=False))
    ms_out = timed(lambda: binding.linear(attn.view(Bsz, N, E), wo[0], out=y))

    cpu = None
    if cpu_baseline:
        # one layer of one image: (b, h) units and images are independent, so the per-image time is exact
        from oracle import dfa_oracle
        wqe = synth.bf16_bits_to_f64(wq_bits[0])
        woe = synth.bf16_bits_to_f64(wo_bits[0])
        t0 = time.perf_counter()
        dfa_oracle.attention_layer(xe[:1], wqe, woe, H, branches, scale)
        dt = time.perf_counter() - t0
        cpu = {"value": dt * layers * 1e6, "unit": "us per image (all layers)", "cores": dfa_oracle.num_threads(),
               "kind": "oracle", "seconds": round(dt, 3),
               "sample": f"one layer of one image in fp64 (numpy matmul projections + the C attention oracle), times {layers} layers"}
    return {
        "metric": f"us per 1024x1024 image, all {layers} layers of the encoder attention stack", "value": wall * 1e6 / Bsz,
        "unit": "us/image", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": wall * 1e3,
        "settle": {"untimed_steps_before_warmup": n_settle},
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"stack: {layers} layers, embed {E}, H={H} D={D}, B={Bsz}, N={N}, branches={branches}, "
                               "QKV projection + dilated attention + output projection per layer"},
        "useful_tflops": flops / wall / 1e12, "pct_of_mfma_peak": 100.0 * flops / wall / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "per_layer_kernels": {
            "qkv_projection": {"ms": ms_qkv, "TFLOP/s": fl_qkv / ms_qkv / 1e9},
            "dilated_attention": {"ms": ms_attn, "TFLOP/s": fl_attn / ms_attn / 1e9},
            "output_projection": {"ms": ms_out, "TFLOP/s": fl_out / ms_out / 1e9}},
        "cpu_baseline": cpu,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200, help="timed steps (default 200)")
    ap.add_argument("--warmup", type=int, default=20, help="untimed steps directly before them (default 20)")
    ap.add_argument("--settle-ms", type=float, default=SETTLE_MS,
                    help="milliseconds of untimed launches back to back before the warm-up steps, so that the timed steps "
                         "run at the chip's steady clock (default %(default)s; 0 times a cold burst)")
    ap.add_argument("--write-traffic", metavar="DIR",
                    help="rewrite profiles/dfa_fwd_hbm_traffic.txt from the counter runs under DIR and exit (no GPU needed)")
    ap.add_argument("--workload", default=WORKLOAD, help="name in synth.CONFIGS (default: throughput)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stack", action="store_true",
                    help="leave the short encoder-attention-stack run out of the default line (profiling runs: the "
                         "stack launches the same kernels on another batch size)")
    ap.add_argument("--stages", action="store_true",
                    help="time the stand-alone stage kernels (gather, placement, unmerged branches, merge) "
                         "on the same workload and print their achieved HBM GB/s instead of the default line")
    ap.add_argument("--stack", action="store_true",
                    help="time the encoder attention stack workload (12 layers of QKV projection + dilated attention "
                         "+ output projection at B = 8) and print its line instead of the default one")
    ap.add_argument("--sweep", action="store_true",
                    help="input-size sweep of the paper's ablation (256^2, 512^2, 1024^2 images; 6 and 12 heads): "
                         "dilated attention against dense attention in the same kernel (w = N, r = 1)")
    ap.add_argument("--sweep-only", type=int, nargs=2, metavar=("SIDE", "HEADS"), default=None,
                    help="with --sweep: only the row of this image side (256, 512 or 1024) and head count (6 or 12)")
    ap.add_argument("--tile-cost", action="store_true",
                    help="single-branch launches of growing segment length on the throughput shape: cost per 64-key "
                         "step and per tile of the forward kernel")
    ap.add_argument("--backward", action="store_true",
                    help="time dfa_backward (dq, dk, dv) on --workload")
    ap.add_argument("--zero-inputs", action="store_true",
                    help="diagnostic: the default line or --backward on all-zero tensors of the same shape (same work, "
                         "no operand bit flips): the gap to the synthetic-data time shows how far the launch is power-limited")
    ap.add_argument("--layers", type=int, default=12, help="--stack: number of layers")
    ap.add_argument("--heads", type=int, default=12, help="--stack: heads of 64 (embed = 64 * heads)")
    ap.add_argument("--batch", type=int, default=None, help="--stack: images per step (default 8; 1 = the latency of one image)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain device-to-device copy of known size (FETCH_SIZE / WRITE_SIZE reference)")
    args = ap.parse_args()
    if args.write_traffic:
        write_traffic(args.write_traffic)
        return
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the path needs no exchange between GPUs: "
                 "(b, h) units are independent, so N GPUs would each run this same kernel on B/N images). "
                 "Run with --gpus 1.")

    import numpy as np
    import torch
    from paper_2403_09195_amd import binding, synth

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    binding.lib()
    torch.cuda.set_device(0)

    if args.copy_calibration:
        # a plain copy kernel of known size: rocprofv3's FETCH_SIZE / WRITE_SIZE for it give the
        # factor between the counters and real HBM bytes
        n = 1 << 28                                   # 256 MiB read + 256 MiB written per copy
        a = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
        b = torch.empty_like(a)
        for _ in range(5):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_each_way": n, "copies": 5}))
        return

    if args.stack:
        print(json.dumps(stack_report(binding, synth, torch, np, args.steps, args.warmup, not args.no_cpu_baseline,
                                      args.layers, args.heads, args.batch)))
        return
    if args.sweep:
        print(json.dumps(sweep_report(binding, synth, torch, np, args.steps, args.warmup, args.sweep_only)))
        return
    if args.tile_cost:
        print(json.dumps(tile_cost_report(binding, synth, torch, np)))
        return

    cfg = synth.CONFIGS[args.workload]
    Bsz, H, N, D, branches = cfg["B"], cfg["H"], cfg["N"], cfg["D"], cfg["branches"]
    scale = 1.0 / (D ** 0.5)
    storage, exact = synth.qkv(cfg["seed"], Bsz, N, H, D, cfg["dtype"])
    if args.zero_inputs:
        storage, exact = tuple(np.zeros_like(a) for a in storage), tuple(np.zeros_like(a) for a in exact)

    def dev(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
        return torch.from_numpy(a).cuda()

    q, k, v = (dev(a) for a in storage)
    out = torch.empty((Bsz, N, H, D), dtype=q.dtype, device="cuda")
    lse = torch.empty((Bsz, H, N), dtype=torch.float32, device="cuda")
    flops = synth.useful_flops(Bsz, H, N, D, branches)
    # what the kernels execute: the plan visits a key that several branches of a row keep once (weighted by its
    # multiplicity), so the executed (query, key) pairs can be fewer than the algorithm's
    plan = binding.plan_describe(Bsz, H, N, branches)
    executed_pairs = Bsz * sum(int(t[2]) * int(plan["segs"][t[3]:t[3] + t[4], 2].sum()) for t in plan["tiles"])
    executed_flops = 4 * D * executed_pairs

    if args.stages:
        print(json.dumps(stage_report(binding, torch, q, k, v, branches, scale, args.steps, args.warmup)))
        return

    if args.backward:
        binding.forward(q, k, v, branches, scale, out=out, lse=lse)
        g = torch.from_numpy(synth.tensor(cfg["seed"], 7, (Bsz, N, H, D), cfg["dtype"])[0]
                             .view(np.int16 if cfg["dtype"] == "bf16" else np.float32)).cuda()
        g = g.view(torch.bfloat16) if cfg["dtype"] == "bf16" else g
        if args.zero_inputs:
            g.zero_()
        steps = max(1, args.steps if cfg["dtype"] == "bf16" else min(args.steps, 20))   # the fp32 path takes tens of ms
        if cfg["dtype"] == "bf16" and args.settle_ms > 0:
            settle(torch, lambda: binding.backward(q, k, v, out, lse, g, branches, scale), args.settle_ms)
        for _ in range(max(1, min(args.warmup, steps))):
            binding.backward(q, k, v, out, lse, g, branches, scale)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(steps):
            binding.backward(q, k, v, out, lse, g, branches, scale)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        pairs = executed_pairs
        # products of 2*D flops per pair: bf16 path 3 (dq kernel) + 4 (dk and dv together), fp32 path 3 + 2 + 3
        executed = pairs * (14 if cfg["dtype"] == "bf16" else 16) * D
        mfma = cfg["dtype"] == "bf16"
        peak = MFMA_BF16_PEAK_TFLOPS if mfma else 157.3
        print(json.dumps({"metric": "dfa_backward ms per step (dq, dk, dv)", "value": ms, "unit": "ms", "steps": steps,
                          "higher_is_better": False, "config": {"workload": args.workload},
                          "dtype": "bf16" if mfma else "f32", "data": "zeros" if args.zero_inputs else "synthetic",
                          "useful_backward_TFLOP/s": 2.5 * flops / ms / 1e9,
                          "roofline": {"bound": "mfma" if mfma else "alu", "achieved": executed / ms / 1e9, "peak": peak,
                                       "unit": "TFLOP/s", "frac": executed / ms / 1e9 / peak,
                                       "note": "executed flops: products of 2*D per visited (query, key) pair (a pair that several branches hold is visited once): 3 in the dq kernel, 4 in the "
                                               "dk/dv kernel (bf16), 3 + 2 + 3 in the fp32 kernels: scores are recomputed in "
                                               "each kernel; useful = 5 products"}}))
        return

    # a launch with few workgroups is split over several workgroups per tile: the caller's workspace for the partial results
    need = binding.workspace_bytes(Bsz, H, N, D, binding.DFA_BF16 if cfg["dtype"] == "bf16" else binding.DFA_F32, branches)
    ws = torch.empty((need,), dtype=torch.uint8, device="cuda") if need else None

    def step():
        binding.forward(q, k, v, branches, scale, out=out, lse=lse, workspace=ws)

    # untimed: the settle phase (steady clocks), then the warm-up steps as asked for; then exactly `steps` timed steps
    n_settle = settle(torch, step, args.settle_ms) if args.settle_ms > 0 else 0
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3
    tflops = flops / (wall / args.steps) / 1e12

    # dominant (only) kernel: mean launch duration from HIP events on the launch stream over `steps` launches, in the
    # same steady state (the calls above are still draining when these are enqueued: no idle gap in between)
    for _ in range(args.warmup):
        step()
    kern_ms = binding.forward_timed(q, k, v, branches, scale, args.steps, out=out, lse=lse, workspace=ws)
    achieved = flops / (kern_ms * 1e-3) / 1e12
    # and launch by launch: events between consecutive launches of one uninterrupted run on that same stream (torch's
    # current stream is the stream the binding launches on); the median of the last 100 of 150
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(151)]
    for i in range(150):
        evs[i].record()
        step()
    evs[150].record()
    torch.cuda.synchronize()
    each = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(50, 150))
    kern_ms_median = 0.5 * (each[49] + each[50])

    # the matrix cores on their own, measured now on this machine: constant and random operands
    peak_const, mhz_const = binding.mfma_peak(False)
    peak_rand, mhz_rand = binding.mfma_peak(True)

    # CPU baseline leg: the oracle as it stands, timed on the host cores on the whole workload; its result also
    # says how far what was just timed is from it (every element of the output)
    cpu = None
    max_err = None
    if not args.no_cpu_baseline:
        from oracle import dfa_oracle
        bs = Bsz                                      # the oracle needs only seconds for the whole batch
        sub = tuple(np.ascontiguousarray(a[:bs]) for a in exact)
        t0 = time.perf_counter()
        o_ref, _ = dfa_oracle.forward(*sub, branches, scale)
        dt = time.perf_counter() - t0
        cpu = {"value": synth.useful_flops(bs, H, N, D, branches) / dt / 1e12, "unit": "TFLOP/s",
               "cores": dfa_oracle.num_threads(), "kind": "oracle", "seconds": round(dt, 3),
               "sample": f"the whole workload: {bs} of {Bsz} images, all {H} heads ({bs * H} independent (b,h) units), fp64"}
        max_err = float(np.abs(out[:bs].float().cpu().numpy().astype(np.float64) - o_ref).max())

    # the second half of the headline metric: one 1024^2 image through all 12 layers of the encoder
    # attention stack (projections included), from a short run of the stack workload
    stack = None
    if args.workload == WORKLOAD and not args.zero_inputs and not args.no_stack:
        try:
            del q, k, v, out, lse
            rep = stack_report(binding, synth, torch, np, 5, 2, False)
            stack = {"us_per_image_all_12_layers": rep["value"], "useful_TFLOP/s": rep["useful_tflops"],
                     "workload": rep["config"]["workload"]}
        except Exception as exc:                      # the main figure must not depend on this extra
            stack = {"error": repr(exc)}

    line = {
        # the metric as the task definition words it; `value` is its first part (useful attention FLOPs, 4*D per
        # kept (query, key) pair), the other two parts are pct_of_mfma_peak and encoder_attention_stack below
        "metric": "dilated-attention TFLOP/s + % MFMA peak; \u00b5s per 1024\u00b2 image (all layers)",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "settle": {"untimed_launches_before_warmup": n_settle, "ms_asked": args.settle_ms,
                   "why": "steady-state figure: a burst of launches starts with a clock transient of some 30 ms"},
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg["dtype"] == "bf16" else "f32",
        "data": "zeros (power diagnostic, not the benchmark)" if args.zero_inputs else "synthetic",
        "config": {"workload": f"{args.workload}: B={Bsz} H={H} N={N} D={D} branches={branches} offset=h mod r scale=1/sqrt(D)"},
        "pct_of_mfma_peak": 100.0 * tflops / MFMA_BF16_PEAK_TFLOPS,
        "mfma_only_loop": {"constant_operands": {"TFLOP/s": peak_const, "shader_MHz": mhz_const},
                           "random_operands": {"TFLOP/s": peak_rand, "shader_MHz": mhz_rand},
                           "pct_of_random_operand_ceiling": 100.0 * tflops / peak_rand},
        "us_per_image_per_layer": ms_per_step * 1e3 / Bsz,
        "us_per_image_12_layers_attention_only": 12 * ms_per_step * 1e3 / Bsz,
        "encoder_attention_stack": stack,
        "useful_flops_per_step": flops,
        "max_abs_err_vs_oracle": max_err,
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": None if args.zero_inputs else read_traffic(args.workload),
                     "algorithmic_bytes": Bsz * N * H * (4 * D * (2 if cfg["dtype"] == "bf16" else 4) + 4),
                     "kernel": "dfa_fwd_bf16_kernel" if cfg["dtype"] == "bf16" else "dfa_fwd_f32_kernel",
                     "kernel_ms": kern_ms, "kernel_ms_median_of_100": kern_ms_median,
                     "executed_flops_per_step": executed_flops,
                     "executed_TFLOP/s": executed_flops / (kern_ms * 1e-3) / 1e12,
                     "mfma_utilisation_executed": executed_flops / (kern_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                     "note": "achieved and frac count the algorithm's flops (4*D per kept (query, key) pair of every branch) "
                             "per launch; the kernel visits a key that several branches of a row keep once, weighted by its "
                             "multiplicity, so the matrix cores execute fewer: executed_* and mfma_utilisation_executed "
                             "count those (the figure to read as how busy the matrix cores are)"},
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
