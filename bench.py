#!/usr/bin/env python3
"""Benchmark of the ELMO head training step on one MI355X.

A step = one pass of the whole hot path (step set-up, then per label chunk: logits + BCE epilogue,
input gradient, fused update -- the last two in one kernel when the batch is at most 128 rows --;
then the finalise kernel) over one fresh synthetic batch that is already resident in HBM.
Default workload: the 3M-label FP8 head, the headline configuration (L = 3,000,000, d = 768, B = 1024, E4M3
weights + BF16 Kahan buffer + stochastic rounding, about 8 Zipf(1.05) positives per sample,
chunk = 131072).

Prints ONE JSON line: samples/s of that workload, plus
  * `roofline` for its dominant kernel: algorithmic flops (2 B n d per product) or algorithmic bytes
    (the read-modify-write of the weights and the compensation, n d (2 s_w + 4 [Kahan]), nothing
    else) per launch over the average launch time, measured with HIP events on the launch stream
    inside the timed region.  The bound is chosen by the regime: the matrix cores when the padded
    batch exceeds 128 rows, HBM bandwidth below; both fractions are printed either way.  What a
    kernel moves beyond the algorithmic bytes because of how the step is split into kernels (the
    logit-gradient buffer, re-reads of W, X) is listed separately as `structure_bytes`;
  * `step_times_ms`: median / min / max over the timed steps (event pairs around every step);
  * `memory`: planned bytes next to torch's measured peak;
  * `small_batch` (default workload only): the same head stepped with B = 128, chunk = 262144,
    the bandwidth regime of the sweep configuration;
  * `topk` (default workload only, or --topk K): elmo_head_topk with k = 100 for the batch;
  * `cpu_baseline`: the FP64 CPU oracle timed on a bounded label sample of the same workload.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import statistics
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
    """HBM-side bytes per launch of `kernel` as recorded in the committed rocprofv3 counter summary
    `profile` under profiles/ (FETCH_SIZE and WRITE_SIZE, scaled by the factors measured in the same
    runs), or None.  Not measured by this run: the caller labels it with its source."""
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
    ap.add_argument("--no-kahan", action="store_true", help="without the compensation buffer")
    ap.add_argument("--kahan-head", type=float, default=None,
                    help="compensation for this fraction of the labels only (the most frequent ones, ids 0..)")
    ap.add_argument("--dropout", type=float, default=0.0, help="classifier dropout rate inside the products (default none)")
    ap.add_argument("--no-dx", action="store_true", help="skip the input gradient (weights-only step)")
    ap.add_argument("--topk", type=int, default=None, help="time elmo_head_topk with this k (default: 100 on the default workload)")
    ap.add_argument("--no-small-batch", action="store_true", help="skip the B = 128 sub-record of the default workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run one plain 1 GiB device copy (a kernel of known traffic for scaling rocprofv3 counters)")
    ap.add_argument("--cpu-sample-labels", type=int, default=131072)
    return ap.parse_args()


def measure(b, synth, torch, np, cfg, args, n_warm, n_steps, dev, profile_name, keep_first_batch=False):
    """Create the head of `cfg`, run n_warm + n_steps steps on fresh batches, return the figures."""
    L, d, B = cfg.L, cfg.d, cfg.B
    fp8 = cfg.fmt == synth.E4M3
    kahan = bool(cfg.flags & synth.FLAG_KAHAN)
    s_w = 1 if fp8 else 2
    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()
    mem_before = torch.cuda.memory_allocated()

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
        del f
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
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(n_steps + 1)]
    b.elmo_head_profile(head.h, True)
    t0 = time.perf_counter()
    marks[0].record(stream)
    for i, s in enumerate(range(n_warm, n_warm + n_steps)):
        run(s)
        marks[i + 1].record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = b.elmo_head_profile_read(head.h)
    b.elmo_head_profile(head.h, False)
    ms_per_step = (t1 - t0) * 1e3 / n_steps
    per_step = [marks[i].elapsed_time(marks[i + 1]) for i in range(n_steps)]
    mem_peak = torch.cuda.max_memory_allocated() - mem_before

    # ---------------- per-kernel algorithmic work (per launch = per chunk; averaged over the chunks)
    n_chunks = -(-L // cfg.chunk)
    n_avg = L / n_chunks                                   # labels per launch, averaged
    Bp = -(-B // 64) * 64
    # padded batches of at most 128 rows take the single-pass kernel: input gradient and update share
    # one launch (timed under "update") and one read of W
    fused = (not args.no_dx) and prof["dx"][1] == 0
    regime = "hbm" if Bp <= 128 else "mfma"
    rmw_bytes = n_avg * d * (2 * s_w + 4 * kahan_frac)    # the weights and the compensation read once, written once
    g_bytes, w_bytes, x_bytes = Bp * n_avg * 2, n_avg * d * s_w, B * d * 2
    kern = {}
    for name, flops, peak_tf, algo_bytes, structure in (
        ("logits", 2.0 * B * n_avg * d, PEAK_FP8_TFLOPS if fp8 else PEAK_BF16_TFLOPS, 0.0, w_bytes + g_bytes + B * d * s_w),
        ("dx", 2.0 * B * n_avg * d, PEAK_BF16_TFLOPS, 0.0, w_bytes + g_bytes),
        ("update", (4.0 if fused else 2.0) * B * n_avg * d, PEAK_BF16_TFLOPS, rmw_bytes, g_bytes + x_bytes),
    ):
        ms, n = prof[name]
        if n == 0:
            continue
        avg_ms = ms / n
        kern[name] = {
            "avg_ms": avg_ms, "launches": int(n), "share_of_step": ms / n_steps / ms_per_step,
            "algorithmic_flops": flops, "tflops": flops / avg_ms * 1e-9, "mfma_peak_tflops": peak_tf,
            "mfma_frac": flops / avg_ms * 1e-9 / peak_tf,
            "algorithmic_bytes": algo_bytes, "algo_gbs": algo_bytes / avg_ms * 1e-6,
            "hbm_frac": algo_bytes / avg_ms * 1e-6 / PEAK_HBM_GBS,
            "structure_bytes": structure,
        }
        if name == "update" and fused:
            kern[name]["includes_input_gradient"] = True
    dom = max(kern, key=lambda k: kern[k]["avg_ms"] * kern[k]["launches"])
    if regime == "hbm":
        dom = "update"                                      # the kernel that carries the weight read-modify-write
    kd = kern[dom]
    if regime == "mfma":
        roof = {"bound": "mfma", "achieved": kd["tflops"], "unit": "TFLOP/s", "peak": kd["mfma_peak_tflops"], "frac": kd["mfma_frac"]}
    else:
        roof = {"bound": "hbm", "achieved": kd["algo_gbs"], "unit": "GB/s", "peak": PEAK_HBM_GBS, "frac": kd["hbm_frac"]}
    traffic = profiled_traffic(dom, profile_name, fused)
    roof.update({"kernel": dom, "avg_launch_ms": kd["avg_ms"], "mfma_frac": kd["mfma_frac"], "hbm_frac": kd["hbm_frac"],
                 "regime_rule": "padded batch <= 128 rows: hbm, above: mfma",
                 "traffic": traffic,
                 "traffic_source": (f"profiles/{profile_name} (rocprofv3 FETCH_SIZE + WRITE_SIZE of an earlier run of this "
                                    "command, not measured by this run)") if traffic else None})

    # whole-step figures of the headline metric: flop/s against the FP8 MFMA peak (6 B L d flop per
    # step, of which 2 B L d can run at the FP8 rate and 4 B L d must run at the BF16 rate) and the
    # weight read-modify-write bytes against HBM peak
    n_prod = 3.0 if not args.no_dx else 2.0
    step_flops = 2.0 * n_prod * B * L * d
    blended_ms = (2.0 * B * L * d / (PEAK_FP8_TFLOPS if fp8 else PEAK_BF16_TFLOPS) + 2.0 * (n_prod - 1) * B * L * d / PEAK_BF16_TFLOPS) * 1e-9
    step_bytes = L * d * (2 * s_w + 4 * kahan_frac)
    whole = {
        "step_tflops": step_flops / ms_per_step * 1e-9,
        "frac_of_fp8_mfma_peak": step_flops / ms_per_step * 1e-9 / PEAK_FP8_TFLOPS,
        "frac_of_blended_mfma_peak": blended_ms / ms_per_step,
        "weight_rmw_gbs": step_bytes / ms_per_step * 1e-6,
        "frac_of_hbm_peak": step_bytes / ms_per_step * 1e-6 / PEAK_HBM_GBS,
    }
    memory = {"W": head.bytes[0], "comp": head.bytes[1], "workspace": head.bytes[2],
              "one_chunk_logit_buffer": b.elmo_logit_buffer_bytes(B, min(cfg.chunk, L)),
              "planned_total": sum(head.bytes),
              "torch_peak_allocated_delta": int(mem_peak),
              "note": "torch's peak also holds the resident batches and the FP32 staging slices of the weight initialisation"}
    res = {
        "samples_per_s": B * n_steps / (t1 - t0), "ms_per_step": ms_per_step,
        "step_times_ms": {"median": statistics.median(per_step), "min": min(per_step), "max": max(per_step), "n": n_steps},
        "roofline": roof, "kernels": kern, "whole_step": whole, "memory": memory,
        "config": {"workload": cfg.name, "L": L, "d": d, "B": B, "chunk": cfg.chunk, "chunks": n_chunks,
                   "weights": "e4m3" if fp8 else "bf16", "kahan_bf16": kahan, "kahan_label_fraction": kahan_frac,
                   "stochastic_rounding": bool(cfg.flags & synth.FLAG_SR),
                   "positives_per_sample": float(len(batches[0][2]) / B), "zipf_s": cfg.zipf_s, "lr": cfg.lr,
                   "input_gradient": not args.no_dx, "classifier_dropout": round(args.dropout * 256) / 256},
    }
    return res, head, batches, kahan_rows


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
            flags = cfg.flags & ~synth.FLAG_KAHAN if args.no_kahan else cfg.flags
            cfg = dataclasses.replace(cfg, B=args.batch or cfg.B, chunk=args.chunk or cfg.chunk, flags=flags)
    default_workload = (args.workload == "xl" and not (args.batch or args.chunk or args.no_kahan or args.no_dx or args.dropout)
                        and args.kahan_head is None)
    L, d, B = cfg.L, cfg.d, cfg.B
    fp8 = cfg.fmt == synth.E4M3
    kahan = bool(cfg.flags & synth.FLAG_KAHAN)

    # committed counter summaries exist for exactly these two workloads
    profile = None
    plain = not args.no_dx and not args.no_kahan and args.kahan_head is None and not args.dropout
    if plain and default_workload:
        profile = "head_step_xl_fp8_B1024.txt"
    elif plain and args.workload == "xl_sweep" and B == 128 and cfg.chunk == 262144:
        profile = "head_step_xl_fp8_B128.txt"

    res, head, batches, kahan_rows = measure(b, synth, torch, np, cfg, args, args.warmup, args.steps, dev, profile)
    stream = torch.cuda.current_stream()

    topk = None
    k_top = args.topk if args.topk is not None else (100 if default_workload else 0)
    if k_top:
        idx = torch.zeros((B, k_top), dtype=torch.int32, device=dev)
        sc = torch.zeros((B, k_top), dtype=torch.float32, device=dev)
        head.topk(batches[0][0], k_top, idx, sc, stream)
        torch.cuda.synchronize()
        reps, times = 5, []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            head.topk(batches[0][0], k_top, idx, sc, stream)
            e1.record(stream)
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1))
        dt = statistics.median(times) * 1e-3
        topk = {"k": k_top, "queries": B, "ms_median": dt * 1e3, "ms_min": min(times), "repeats": reps, "queries_per_s": B / dt,
                "frac_of_mfma_peak": 2.0 * B * L * d / dt * 1e-12 / (PEAK_FP8_TFLOPS if fp8 else PEAK_BF16_TFLOPS)}
        del idx, sc

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
        Wb = head.weights()[:n_s].cpu().numpy()
        Wb = Wb.view(np.uint16) if not fp8 else Wb
        Cb = np.zeros((n_s, d), np.uint16) if kahan else None
        t2 = time.perf_counter()
        o.head_step(Wb, Cb, X0, ip0, ix0, cfg.lr, 0, 0, cfg.fmt, cfg.flags, label_ids=np.arange(n_s),
                    kahan_rows=(kahan_rows or None) if kahan else None, dropout=int(round(args.dropout * 256)))
        dt = time.perf_counter() - t2
        how = "all labels, nothing extrapolated" if n_s == L else f"extrapolated x{L / n_s:.1f} to all labels"
        cpu = {"value": B / (dt * L / n_s), "unit": "samples/s", "cores": int(cores), "kind": "oracle",
               "sample": f"one full oracle step (FP64 logits, gradients, update with the same Philox fields) on labels "
                         f"0..{n_s - 1} of {L} with the full batch of {B}: {dt:.2f} s, {how}"}

    head.close()
    del head, batches
    torch.cuda.empty_cache()

    small = None
    if default_workload and not args.no_small_batch:
        cfg_s = synth.xl_sweep(128, 262144, True)
        r, h2, b2, _ = measure(b, synth, torch, np, cfg_s, args, 3, 10, dev, "head_step_xl_fp8_B128.txt")
        h2.close()
        del h2, b2
        small = {"config": r["config"], "value": r["samples_per_s"], "unit": "samples/s", "ms_per_step": r["ms_per_step"],
                 "steps": 10, "warmup": 3, "step_times_ms": r["step_times_ms"], "roofline": r["roofline"], "kernels": r["kernels"],
                 "whole_step": r["whole_step"]}

    out = {
        "metric": "head train samples/s + MFMA% / HBM% of peak at 3M labels, d=768, fp8" if args.workload.startswith("xl")
                  else "head train samples/s",
        "value": res["samples_per_s"], "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8" if fp8 else "bf16",
        "data": "synthetic",
        "config": res["config"],
        "roofline": res["roofline"], "step_times_ms": res["step_times_ms"], "kernels": res["kernels"],
        "whole_step": res["whole_step"], "memory": res["memory"], "cpu_baseline": cpu,
    }
    if topk:
        out["topk"] = topk
    if small:
        out["small_batch"] = small
    print(json.dumps(out))


if __name__ == "__main__":
    main()
