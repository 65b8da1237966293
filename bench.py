#!/usr/bin/env python3
"""Benchmark of the head-selective ViT block stack on one MI355X.

One step = forward through all blocks, then backward through all blocks (every
row of the hot path: LayerNorms, QKV / attention / output projection over the
live heads, MLP, and the backward kernels for p_f heads), on seeded synthetic
token batches that are resident in HBM before the timed region.

Prints ONE JSON line: images/s for the configured head-op mask, the all-full
mask beside it, the roofline of the dominant kernel (measured live with HIP
events inside the library) and the CPU oracle timed on the host cores.
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

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
# the metric as the baseline record names it; the headline line is the ViT-B/16 stack with 60 % p_f / 20 % p_o /
# 20 % p_s heads, and the literal "40 % of the heads skipped" mask is the sub-record "vit_b16_skip40"
METRIC = "fine-tune step images/sec, ViT-B/16 block stack, 40% heads skipped; MFMA util %"


def algorithmic_flops(w, ops, rows=None) -> float:
    """FLOPs one step must do: skipped heads and the backward of non-full heads are not counted."""
    import d2ft_inputs as di
    M, D, T, dh, Dm, r = (w.rows if rows is None else rows), w.width, w.tokens, w.head_dim, w.mlp_hidden, w.lora_rank
    total = 0.0
    for l in range(ops.shape[0]):
        n_full = int((ops[l] == di.OP_FULL).sum())
        n_live = n_full + int((ops[l] == di.OP_FWD).sum())
        head_fwd = 4.0 * M * dh * (2 * D + T)
        if w.gate_ffn:   # whole subnets: each head carries Dm/H hidden units
            head_fwd += 4.0 * M * D * (Dm // w.heads)
            total += (n_live + 2 * n_full) * head_fwd
        elif w.train_base:
            total += (n_live + 2 * n_full) * head_fwd + 12.0 * M * D * Dm
        else:   # LoRA: no base weight gradients
            lora_fwd = 4.0 * M * r * (D + dh)
            total += n_live * (head_fwd + lora_fwd)
            total += n_full * (8.0 * M * dh * (D + T) + 8.0 * M * r * (D + dh))
            total += 8.0 * M * D * Dm
    return total


def recorded_traffic(kernel: str, workload: str):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary, or None when the
    summary is for another kernel / workload or the kernel source has changed since it was taken."""
    import hashlib
    path = os.path.join(ROOT, "profiles", "gemm_hbm_traffic_vit_b16.txt")
    src = os.path.join(ROOT, "paper_2504_12471_amd", "csrc", "kernels_gemm_mfma.hip")
    try:
        rec = None
        for line in open(path):
            if line.startswith("{"):
                rec = json.loads(line)
        if rec is None or rec["workload"] != workload or kernel not in rec["kernels"]:
            return None
        if hashlib.sha256(open(src, "rb").read()).hexdigest() != rec["source_sha256"]:
            return None
        k = rec["kernels"][kernel]
        return {"bytes_per_launch": k["bytes_per_launch"], "fetch_bytes": k["fetch_bytes"],
                "write_bytes": k["write_bytes"], "unit": "B"}
    except (OSError, KeyError, ValueError):
        return None


def sub_records(args, w, s, dws, x, dy, grad_fields):
    """The ViT-B/16 stack under the other masks and modes, same weights and token batch, timed in the same run:
    the metric's literal mask (40 % of the heads skipped, none forward-only), whole subnets gated (a head
    with its 1/H slice of the feed-forward network, Sec. II-A.1), and one op code per (subnet, micro-batch)
    with 5 micro-batches (Alg. 1's table; Sec. III-A), each with its all-p_f time and FLOP ratio."""
    import numpy as np
    import torch

    import d2ft_inputs as di
    import paper_2504_12471_amd as P

    steps, warmup = max(10, args.steps // 2), max(3, args.warmup // 4)

    def timed(stack, mask):
        for _ in range(warmup):
            stack.step(x, dy, mask)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            stack.step(x, dy, mask)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    def record(name, wl, ops, mb_images):
        desc = P.make_desc(wl.batch, wl.tokens, wl.width, wl.heads, wl.mlp_hidden, wl.dtype, wl.lora_rank, wl.lora_scale,
                           wl.ln_eps, wl.head_dim, P.FLAG_GATE_FFN if wl.gate_ffn else 0)
        stack = P.BlockStack(desc, dws, wl.dtype, grad_fields, mb_images)
        ms = timed(stack, ops)
        ms_full = timed(stack, np.full_like(ops, di.OP_FULL))
        if mb_images is None:
            fl = algorithmic_flops(wl, ops)
            fl_full = algorithmic_flops(wl, np.full_like(ops, di.OP_FULL))
        else:
            fl = sum(algorithmic_flops(wl, ops[:, i], mb_images[i] * wl.tokens) for i in range(len(mb_images)))
            fl_full = algorithmic_flops(wl, np.full_like(ops[:, 0], di.OP_FULL))
        del stack
        torch.cuda.empty_cache()
        return {"workload": name, "ms_per_step": round(ms, 4), "images_per_s": round(wl.batch / (ms * 1e-3), 1),
                "all_full_ms_per_step": round(ms_full, 4), "time_ratio": round(ms / ms_full, 4),
                "flop_ratio": round(fl / fl_full, 4), "step_mfma_frac": round(fl / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                "heads_full": int((ops == di.OP_FULL).sum()), "heads_fwd_only": int((ops == di.OP_FWD).sum()),
                "heads_skipped": int((ops == di.OP_SKIP).sum()), "micro_batches": mb_images, "steps": steps}

    out = []
    for name in ("vit_b16_skip40", "vit_b16_ffn", "vit_b16_ffn_skip40"):
        wl = di.WORKLOADS[name]
        out.append(record(name, wl, di.draw_ops(wl, args.seed)[0], None))
    base, extra = divmod(w.batch, 5)
    mb = [base + (1 if i < extra else 0) for i in range(5)]
    for name in ("vit_b16", "vit_b16_ffn"):
        wl = di.WORKLOADS[name]
        rng = np.random.default_rng(args.seed + 1000)
        ops = di.exact_count_masks(rng, wl.blocks * 5, wl.heads, *wl.mask[1:]).reshape(wl.blocks, 5, wl.heads)
        out.append(record(name + " --micro 5", wl, ops, mb))
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="vit_b16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-all-full", action="store_true")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--micro", type=int, default=0,
                    help="split the batch into this many micro-batches, each with its own op codes (0: one code per head)")
    ap.add_argument("--no-sub-records", action="store_true",
                    help="skip the extra workloads timed beside the headline one (skip40 mask, gated FFN, 5 micro-batches)")
    ap.add_argument("--one-stream", action="store_true",
                    help="every launch on the caller's stream (D2FT_FLAG_ONE_STREAM): for kernel traces in which each "
                         "kernel runs alone; the default lets the backward's weight-gradient work run on a second stream")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for scaling HBM traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on ONE GPU (one device's head share, no collectives); --gpus must be 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import d2ft_inputs as di
    import paper_2504_12471_amd as P

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    w = di.WORKLOADS[args.workload]
    s = di.draw_stack(w, args.seed)
    if s.ops is None:   # op codes chosen by the bi-level knapsack on the GPU
        ks = s.knapsack
        codes = P.d2ft_select_knapsack(ks.score_full, ks.score_fwd, ks.cost_fwd, ks.cost_bwd, ks.cap_full, ks.cap_fwd)
        ops = codes.reshape(w.blocks, w.heads)
    else:
        ops = s.ops
    full_ops = di.all_full_ops(w)

    desc = P.make_desc(w.batch, w.tokens, w.width, w.heads, w.mlp_hidden, w.dtype, w.lora_rank, w.lora_scale,
                       w.ln_eps, w.head_dim, (P.FLAG_GATE_FFN if w.gate_ffn else 0) | (P.FLAG_ONE_STREAM if args.one_stream else 0))
    dws = [{k: P.to_device(v, w.dtype) for k, v in bw.items()} for bw in s.weights]
    if w.train_base:
        grad_fields = [k for k in P.WEIGHT_FIELDS if not k.startswith("ln")]   # norm layers frozen (Sec. III-A)
    else:
        grad_fields = ["lora_a_q", "lora_a_v", "lora_b_q", "lora_b_v"]
    mb_images = None
    if args.micro > 0:
        # one code per (subnet, micro-batch) (Alg. 1, T_opt[k][x_i]); the same mask recipe over all of them
        base, extra = divmod(w.batch, args.micro)
        mb_images = [base + (1 if i < extra else 0) for i in range(args.micro)]
        if w.mask[0] != "counts" or base < 1:
            print("bench.py: --micro needs a counts mask and at least one image per micro-batch", file=sys.stderr)
            return 2
        rng = np.random.default_rng(args.seed + 1000)
        ops = di.exact_count_masks(rng, w.blocks * args.micro, w.heads, *w.mask[1:]).reshape(
            w.blocks, args.micro, w.heads)
        full_ops = np.full_like(ops, di.OP_FULL)
    stack = P.BlockStack(desc, dws, w.dtype, grad_fields, mb_images)
    x, dy = P.to_device(s.x, w.dtype), P.to_device(s.dy, w.dtype)

    # step time measured the same with 3 and with 100 warm-up steps; the default of 20 is margin
    def timed(mask, steps, warmup, stack=stack):
        for _ in range(warmup):
            stack.step(x, dy, mask)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            stack.step(x, dy, mask)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    if args.calibration_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    ms = timed(ops, args.steps, args.warmup)
    ms_full = None if args.no_all_full else timed(full_ops, args.steps, min(args.warmup, 20))
    # the same step with every launch on one stream: the launch order the per-kernel figures below are taken in
    ms_one = None
    if not args.no_all_full and not args.one_stream and w.dtype == "bf16":
        desc_one = P.make_desc(w.batch, w.tokens, w.width, w.heads, w.mlp_hidden, w.dtype, w.lora_rank, w.lora_scale,
                               w.ln_eps, w.head_dim, (P.FLAG_GATE_FFN if w.gate_ffn else 0) | P.FLAG_ONE_STREAM)
        stack_one = P.BlockStack(desc_one, dws, w.dtype, grad_fields, mb_images)
        ms_one = timed(ops, max(10, args.steps // 2), min(args.warmup, 10), stack_one)
        del stack_one

    # per-kernel durations, measured with HIP events inside the library on the launch stream
    stack.step(x, dy, ops)
    torch.cuda.synchronize()
    P.d2ft_timing_enable(True)
    n_prof = 10
    for _ in range(n_prof):
        stack.step(x, dy, ops)
    torch.cuda.synchronize()
    kern = P.d2ft_timing_read(64)
    # contribution-score kernels (Sec. II-B): Fisher scores of every block's gradients, timed the same way
    P.d2ft_timing_enable(True)
    for l in range(w.blocks):
        P.d2ft_subnet_scores(desc, stack.grads[l], P.SCORE_FISHER)
    sc = [k for k in P.d2ft_timing_read(8) if "scores" in k["name"]]
    P.d2ft_timing_enable(False)
    head_bytes = sum(t.numel() * t.element_size() for k, t in stack.grads[0].items()
                     if t is not None and (k in ("w_qkv", "b_qkv", "w_o") or k.startswith("lora")
                                           or (w.gate_ffn and k in ("w1", "b1", "w2"))))
    # optimizer step (Sec. IV-A: SGD with momentum) on every block, slices of the p_f subnets only
    mom = [{k: (None if t is None else torch.zeros(t.shape, dtype=torch.float32, device="cuda"))
            for k, t in stack.grads[l].items()} for l in range(w.blocks)]
    step_ops = ops if mb_images is None else np.where((ops == di.OP_FULL).any(axis=1), di.OP_FULL, di.OP_SKIP)
    P.d2ft_timing_enable(True)
    for l in range(w.blocks):
        P.d2ft_sgd_step(desc, dws[l], stack.grads[l], mom[l], None, step_ops[l], 0.0, 0.9, 0.0)   # lr 0: weights keep their values
    torch.cuda.synchronize()
    sg = [k for k in P.d2ft_timing_read(8) if "sgd" in k["name"]]
    P.d2ft_timing_enable(False)
    sgd = None
    if sg:
        es = 2 if w.dtype == "bf16" else 4
        elems = 0
        for l in range(w.blocks):
            for k, t in stack.grads[l].items():
                if t is None:
                    continue
                per_head = k in ("w_qkv", "b_qkv", "w_o") or k.startswith("lora") or (w.gate_ffn and k in ("w1", "b1", "w2"))
                frac = float((step_ops[l] == di.OP_FULL).mean()) if per_head else 1.0
                elems += t.numel() * frac
        sgd_ms = sum(k["ms"] for k in sg)
        sgd = {"ms_per_step": round(sgd_ms, 4), "bytes_per_step": int(elems * (3 * es + 8)),
               "GB_per_s": round(elems * (3 * es + 8) / (sgd_ms * 1e-3) / 1e9, 1)}
    del mom
    scores = None
    if sc:
        us = sc[0]["ms"] / sc[0]["launches"] * 1e3
        scores = {"kind": "fisher", "us_per_block": round(us, 2), "bytes_per_block": head_bytes,
                  "GB_per_s": round(head_bytes / (us * 1e-6) / 1e9, 1)}
    kern.sort(key=lambda k: -k["ms"])
    total_kernel_ms = sum(k["ms"] for k in kern) / n_prof
    dom = kern[0]
    dom_tflops = dom["flops"] / (dom["ms"] * 1e-3) / 1e12 if dom["flops"] > 0 else 0.0
    gemm_ms = sum(k["ms"] for k in kern if k["flops"] > 0)
    gemm_fl = sum(k["flops"] for k in kern if k["flops"] > 0)
    traffic = recorded_traffic(dom["name"], w.name)
    roofline = {
        "bound": "mfma", "kernel": dom["name"], "achieved": round(dom_tflops, 1), "peak": PEAK_BF16_TFLOPS,
        "unit": "TFLOP/s", "frac": round(dom_tflops / PEAK_BF16_TFLOPS, 4),
        "traffic": None if traffic is None else traffic["bytes_per_launch"], "traffic_detail": traffic,
        "avg_launch_us": round(dom["ms"] / dom["launches"] * 1e3, 2), "launches_per_step": dom["launches"] // n_prof,
        "all_gemm_kernels_tflops": round(gemm_fl / (gemm_ms * 1e-3) / 1e12, 1) if gemm_ms > 0 else None,
    }
    kernels = [{"name": k["name"], "launches_per_step": k["launches"] // n_prof,
                "ms_per_step": round(k["ms"] / n_prof, 4),
                "tflops": round(k["flops"] / (k["ms"] * 1e-3) / 1e12, 1) if k["flops"] > 0 else None} for k in kern]
    # bandwidth-bound kernels: algorithmic bytes (every operand read once, every result written once) over the
    # HIP-event time; operands of up to 78 MB can sit in the 256 MB last-level cache
    hbm_kernels = [{"name": k["name"], "launches_per_step": k["launches"] // n_prof,
                    "us_per_launch": round(k["ms"] / k["launches"] * 1e3, 2),
                    "MB_per_launch": round(k["bytes"] / k["launches"] / 1e6, 2),
                    "GB_per_s": round(k["bytes"] / (k["ms"] * 1e-3) / 1e9, 1),
                    "frac_of_hbm_peak": round(k["bytes"] / (k["ms"] * 1e-3) / 1e9 / PEAK_HBM_GBS, 3)}
                   for k in kern if k["bytes"] > 0]

    if mb_images is None:
        flops = algorithmic_flops(w, ops)
    else:
        flops = sum(algorithmic_flops(w, ops[:, i], mb_images[i] * w.tokens) for i in range(args.micro))
    out = {
        "metric": METRIC,
        "value": round(w.batch / (ms * 1e-3), 1), "unit": "images/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic (seeded N(0,1) tokens, N(0,0.02^2) weights)",
        "config": {"workload": w.name, "batch": w.batch, "tokens": w.tokens, "width": w.width, "heads": w.heads,
                   "mlp_hidden": w.mlp_hidden, "blocks": w.blocks, "lora_rank": w.lora_rank, "gate_ffn": w.gate_ffn,
                   "micro_batches": mb_images, "heads_full": int((ops == di.OP_FULL).sum()), "heads_fwd_only": int((ops == di.OP_FWD).sum()),
                   "heads_skipped": int((ops == di.OP_SKIP).sum())},
        "algorithmic_tflop_per_step": round(flops / 1e12, 3),
        "step_mfma_frac": round(flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "all_full": None if ms_full is None else {
            "ms_per_step": round(ms_full, 4), "images_per_s": round(w.batch / (ms_full * 1e-3), 1),
            "masked_over_all_full_time": round(ms / ms_full, 4)},
        "one_stream_ms_per_step": None if ms_one is None else round(ms_one, 4),
        "kernel_ms_per_step_sum": round(total_kernel_ms, 4),
        "roofline": roofline,
        "subnet_scores": scores,
        "sgd_step": sgd,
        "hbm_kernels": hbm_kernels,
        "kernels": kernels,
    }
    if args.workload == "vit_b16" and args.micro == 0 and not args.no_sub_records:
        del stack   # its saved-activation buffers
        torch.cuda.empty_cache()
        out["sub_records"] = sub_records(args, w, s, dws, x, dy, grad_fields)

    if not args.no_cpu_baseline:
        # the oracle as it stands, on the host cores: block 0 of the same workload, forward + backward
        from oracle import d2ft_oracle as orc
        cores = os.cpu_count() or 1
        try:
            cores = len(os.sched_getaffinity(0))
        except Exception:
            pass
        cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
        t0 = time.perf_counter()
        n_done = 0
        while n_done < w.blocks and time.perf_counter() - t0 < 12.0:   # a bounded sample: about 12 s of CPU work
            if mb_images is None:
                y, cache = orc.block_fwd(s.weights[n_done], ops[n_done], s.x, w.head_dim, w.ln_eps, w.lora_scale,
                                         gate_ffn=w.gate_ffn)
                orc.block_bwd(s.weights[n_done], cache, s.dy)
            else:
                y, caches = orc.block_fwd_mb(s.weights[n_done], ops[n_done], mb_images, s.x, w.head_dim, w.ln_eps,
                                             w.lora_scale, gate_ffn=w.gate_ffn)
                orc.block_bwd_mb(s.weights[n_done], caches, mb_images, s.dy)
            n_done += 1
        t_block = (time.perf_counter() - t0) / n_done
        out["cpu_baseline"] = {
            "value": round(w.batch / (t_block * w.blocks), 3), "unit": "images/s", "cores": cores, "kind": "oracle",
            "sample": f"blocks 0..{n_done - 1} of {w.blocks} at full shape with their own op codes, fp64 numpy, "
                      f"forward+backward of each once on the same token batch ({t_block:.1f} s per block); "
                      f"step time extrapolated as {w.blocks} x the mean"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
