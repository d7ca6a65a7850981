#!/usr/bin/env python3
"""Benchmark of the ELMO head training step on one MI355X.

A step = one pass of the whole hot path (step set-up, then per label chunk: logits + BCE epilogue,
input gradient, fused update -- one kernel for both when the batch is at most 128 rows --; then
the finalise kernel) over one fresh synthetic batch that is
already resident in HBM.  Default workload: the 3M-label FP8 head of the benchmark spec
(L = 3,000,000, d = 768, B = 1024, E4M3 weights + BF16 Kahan buffer + stochastic rounding,
about 8 Zipf(1.05) positives per sample, chunk = 131072).

Prints ONE JSON line: samples/s, plus `roofline` for the dominant kernel (per-launch time measured
with HIP events on the launch stream inside the timed region) and `cpu_baseline` (the FP64 CPU
oracle timed on a bounded label sample of the same workload, extrapolated to all labels).
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

# MI355X published peaks
PEAK_HBM_GBS = 8000.0
PEAK_BF16_TFLOPS = 2500.0
PEAK_FP8_TFLOPS = 5000.0


def profiled_traffic(kernel: str, profile: str | None, fused: bool = False):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary `profile` under
    profiles/ (FETCH_SIZE and WRITE_SIZE, scaled by the factors measured in the same runs), or None."""
    if profile is None:
        return None
    path = os.path.join(ROOT, "profiles", profile)
    try:
        lines = open(path).read().splitlines()
    except OSError:
        return None
    scale = {}
    for ln in lines:
        ln = ln.strip()
        if ln.startswith("FETCH_SIZE:") or ln.startswith("WRITE_SIZE:"):
            scale[ln.split(":")[0]] = float(ln.rsplit("by", 1)[1])
    name = {"logits": "k_logits", "dx": "k_dx", "update": "k_dx_update" if fused else "k_update"}[kernel]
    for ln in lines:
        f = ln.split()
        if len(f) >= 4 and f[0].startswith(name + "<") and "FETCH" not in ln:
            try:
                fetch_kib, write_kib = float(f[-2]), float(f[-1])
            except ValueError:
                continue
            if len(scale) == 2 and fetch_kib > 1000:       # the counter table, not the timing table
                return (fetch_kib * scale["FETCH_SIZE"] + write_kib * scale["WRITE_SIZE"]) * 1024.0
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="xl", help="tiny | mid | large | xl | xl_sweep")
    ap.add_argument("--batch", type=int, default=None, help="override B (xl_sweep: 32 / 128 / 4096)")
    ap.add_argument("--chunk", type=int, default=None, help="override the label chunk")
    ap.add_argument("--no-kahan", action="store_true", help="xl_sweep without the compensation buffer")
    ap.add_argument("--kahan-head", type=float, default=None,
                    help="compensation for this fraction of the labels only (the most frequent ones, ids 0..)")
    ap.add_argument("--dropout", type=float, default=0.0, help="classifier dropout rate inside the products (default none)")
    ap.add_argument("--no-dx", action="store_true", help="skip the input gradient (weights-only step)")
    ap.add_argument("--topk", type=int, default=0, help="also time elmo_head_topk with this k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run one plain 1 GiB device copy (a kernel of known traffic for scaling rocprofv3 counters)")
    ap.add_argument("--cpu-sample-labels", type=int, default=131072)
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the head shards by label across GPUs by design, "
              "but no multi-GPU path is built); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2510_11168_amd import binding as b
    from paper_2510_11168_amd import synth

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    dev = "cuda:0"
    torch.cuda.set_device(0)

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.workload == "xl_sweep":
        cfg = synth.xl_sweep(args.batch or 128, args.chunk or 65536, not args.no_kahan)
    else:
        cfg = synth.CONFIGS[args.workload]
        if args.batch or args.chunk or args.no_kahan:
            import dataclasses
            flags = cfg.flags & ~synth.FLAG_KAHAN if args.no_kahan else cfg.flags
            cfg = dataclasses.replace(cfg, B=args.batch or cfg.B, chunk=args.chunk or cfg.chunk, flags=flags)
    L, d, B = cfg.L, cfg.d, cfg.B
    fp8 = cfg.fmt == synth.E4M3
    kahan = bool(cfg.flags & synth.FLAG_KAHAN)
    n_steps, n_warm = args.steps, args.warmup

    # ---------------- head + weights (N(0, 0.02) drawn on the device, rounded by the library)
    kahan_rows = 0
    if kahan and args.kahan_head is not None:
        kahan_rows = min(L, max(128, int(round(args.kahan_head * L / 128.0)) * 128))
    kahan_frac = (kahan_rows or L) / L if kahan else 0.0      # share of the labels that carry compensation
    head = b.Head(L, d, cfg.fmt, cfg.chunk, cfg.flags, B, 64 * B, device=dev, kahan_rows=kahan_rows, dropout_p=args.dropout)
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    W = head.weights()
    for l0 in range(0, L, 65536):
        l1 = min(L, l0 + 65536)
        f = torch.randn((l1 - l0) * d, device=dev, generator=g) * cfg.w_std
        b.elmo_quantize(f, f.numel(), cfg.fmt, 0, 0, 0, 0, W[l0:l1])
    torch.cuda.synchronize()

    # ---------------- a fresh batch per step, generated up front and resident in HBM
    zipf = synth.ZipfLabels(L, cfg.zipf_s)
    batches = []
    for s in range(n_warm + n_steps):
        X, indptr, indices = synth.make_batch(cfg, s, zipf)
        batches.append((torch.from_numpy(X.view(np.int16)).to(dev), torch.from_numpy(indptr).to(dev),
                        torch.from_numpy(indices).to(dev), (X, indptr, indices) if s == 0 else None))
    dX = None if args.no_dx else torch.zeros((B, d), dtype=torch.int16, device=dev)
    stream = torch.cuda.current_stream()

    def run(s):
        Xd, ip, ix, _ = batches[s]
        head.step(Xd, ip, ix, cfg.lr, 0, s, dX, None, stream)

    for s in range(n_warm):
        run(s)
    torch.cuda.synchronize()
    b.elmo_head_profile(head.h, True)
    t0 = time.perf_counter()
    for s in range(n_warm, n_warm + n_steps):
        run(s)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = b.elmo_head_profile_read(head.h)
    b.elmo_head_profile(head.h, False)
    ms_per_step = (t1 - t0) * 1e3 / n_steps
    samples_per_s = B * n_steps / (t1 - t0)

    # ---------------- per-kernel algorithmic work (per launch = per chunk; averaged over the chunks)
    n_chunks = -(-L // cfg.chunk)
    n_avg = L / n_chunks                                   # labels per launch, averaged
    s_w = 1 if fp8 else 2
    # padded batches of at most 128 rows take the single-pass kernel: input gradient and update share
    # one launch (timed under "update") and one read of W
    fused = (not args.no_dx) and prof["dx"][1] == 0
    kern = {}
    for name, flops, byts, peak_tf in (
        ("logits", 2.0 * B * n_avg * d, n_avg * d * s_w + B * n_avg * 2 + B * d * s_w, PEAK_FP8_TFLOPS if fp8 else PEAK_BF16_TFLOPS),
        ("dx", 2.0 * B * n_avg * d, n_avg * d * s_w + B * n_avg * 2, PEAK_BF16_TFLOPS),
        ("update", (4.0 if fused else 2.0) * B * n_avg * d, n_avg * d * (2 * s_w + 4 * kahan_frac) + B * n_avg * 2 + B * d * 2,
         PEAK_BF16_TFLOPS),
    ):
        ms, n = prof[name]
        if n == 0:
            continue
        avg_ms = ms / n
        kern[name] = {
            "avg_ms": avg_ms, "launches": int(n), "share_of_step": ms / n_steps / ms_per_step,
            "tflops": flops / avg_ms * 1e-9, "mfma_frac": flops / avg_ms * 1e-9 / peak_tf,
            "algo_gbs": byts / avg_ms * 1e-6, "hbm_frac": byts / avg_ms * 1e-6 / PEAK_HBM_GBS,
        }
        if name == "update" and fused:
            kern[name]["includes_input_gradient"] = True
    dom = max(kern, key=lambda k: kern[k]["avg_ms"] * kern[k]["launches"])
    kd = kern[dom]
    if kd["mfma_frac"] >= kd["hbm_frac"]:
        roof = {"bound": "mfma", "achieved": kd["tflops"], "unit": "TFLOP/s",
                "peak": (PEAK_FP8_TFLOPS if (dom == "logits" and fp8) else PEAK_BF16_TFLOPS), "frac": kd["mfma_frac"]}
    else:
        roof = {"bound": "hbm", "achieved": kd["algo_gbs"], "unit": "GB/s", "peak": PEAK_HBM_GBS, "frac": kd["hbm_frac"]}
    # committed counter summaries exist for exactly these two workloads
    profile = None
    if not args.no_dx and not args.no_kahan and args.kahan_head is None and not args.dropout:
        if args.workload == "xl" and not (args.batch or args.chunk):
            profile = "head_step_xl_fp8_B1024.txt"
        elif args.workload == "xl_sweep" and B == 128 and cfg.chunk == 262144:
            profile = "head_step_xl_fp8_B128.txt"
    roof.update({"kernel": dom, "avg_launch_ms": kd["avg_ms"], "traffic": profiled_traffic(dom, profile, fused)})

    # whole-step figures of the headline metric: flop/s against the FP8 MFMA peak (6 B L d flop per
    # step) and weight read-modify-write bytes against HBM peak
    step_flops = (6.0 if not args.no_dx else 4.0) * B * L * d
    step_bytes = L * d * (2 * s_w + 4 * kahan_frac)
    whole = {
        "step_tflops": step_flops / ms_per_step * 1e-9,
        "frac_of_fp8_mfma_peak": step_flops / ms_per_step * 1e-9 / PEAK_FP8_TFLOPS,
        "weight_rmw_gbs": step_bytes / ms_per_step * 1e-6,
        "frac_of_hbm_peak": step_bytes / ms_per_step * 1e-6 / PEAK_HBM_GBS,
        "head_bytes": {"W": head.bytes[0], "comp": head.bytes[1], "workspace": head.bytes[2],
                       "one_chunk_logit_buffer": b.elmo_logit_buffer_bytes(B, min(cfg.chunk, L))},
    }

    topk = None
    if args.topk:
        idx = torch.zeros((B, args.topk), dtype=torch.int32, device=dev)
        sc = torch.zeros((B, args.topk), dtype=torch.float32, device=dev)
        head.topk(batches[0][0], args.topk, idx, sc, stream)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        reps = 3
        for _ in range(reps):
            head.topk(batches[0][0], args.topk, idx, sc, stream)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t2) / reps
        topk = {"k": args.topk, "ms": dt * 1e3, "queries_per_s": B / dt,
                "frac_of_mfma_peak": 2.0 * B * L * d / dt * 1e-12 / (PEAK_FP8_TFLOPS if fp8 else PEAK_BF16_TFLOPS)}

    # ---------------- the CPU oracle on a bounded label sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import elmo_oracle as o
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        n_s = min(L, args.cpu_sample_labels)
        X0, ip0, ix0 = batches[0][3]
        Wb = W[:n_s].cpu().numpy()
        Wb = Wb.view(np.uint16) if not fp8 else Wb
        Cb = np.zeros((n_s, d), np.uint16) if kahan else None
        t2 = time.perf_counter()
        o.head_step(Wb, Cb, X0, ip0, ix0, cfg.lr, 0, 0, cfg.fmt, cfg.flags, label_ids=np.arange(n_s),
                    kahan_rows=(kahan_rows or None) if kahan else None, dropout=int(round(args.dropout * 256)))
        dt = time.perf_counter() - t2
        cpu = {"value": B / (dt * L / n_s), "unit": "samples/s", "cores": int(cores), "kind": "oracle",
               "sample": f"one full oracle step (FP64 logits, gradients, update with the same Philox fields) on labels "
                         f"0..{n_s - 1} of {L} with the full batch of {B}: {dt:.2f} s, extrapolated x{L / n_s:.1f} to all labels"}

    out = {
        "metric": "head train samples/s + MFMA% / HBM% of peak at 3M labels, d=768, fp8" if args.workload.startswith("xl")
                  else "head train samples/s",
        "value": samples_per_s, "unit": "samples/s", "n_gpus": 1, "steps": n_steps, "warmup": n_warm,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8" if fp8 else "bf16",
        "data": "synthetic",
        "config": {"workload": cfg.name, "L": L, "d": d, "B": B, "chunk": cfg.chunk, "chunks": n_chunks,
                   "weights": "e4m3" if fp8 else "bf16", "kahan_bf16": kahan, "kahan_label_fraction": kahan_frac,
                   "stochastic_rounding": bool(cfg.flags & synth.FLAG_SR),
                   "positives_per_sample": float(len(batches[0][2]) / B), "zipf_s": cfg.zipf_s, "lr": cfg.lr,
                   "input_gradient": not args.no_dx, "classifier_dropout": round(args.dropout * 256) / 256},
        "roofline": roof, "kernels": kern, "whole_step": whole, "cpu_baseline": cpu,
    }
    if topk:
        out["topk"] = topk
    print(json.dumps(out))


if __name__ == "__main__":
    main()
