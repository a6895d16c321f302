#!/usr/bin/env python3
"""Benchmark of the sampled-SGD FastTucker step on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C2]

W warm-up steps, then exactly K timed steps between two events on the library's stream (before the warm-up,
untimed steps are run for --spin-up-seconds of wall time so that the clocks are up; they are reported as
`spin_up_steps`).  A "step" is one pass of the whole hot path over one sample set Psi:
ftk_sample (Philox positions + COO fetch) followed by ftk_sgd_step (row gather, projections,
leave-one-out products, both gradients, both updates).  Inputs are resident in HBM before the
timed region.  Prints ONE JSON line; `value` is sampled nonzeros per second.

The `roofline` object is for the kernel with the largest average duration, timed live with HIP
events on the library's stream (a second timed pass of K steps with per-kernel events).  The
`cpu_baseline` object is the CPU oracle, single-threaded, on a bounded number of the same steps.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
FP32_MFMA_PEAK_TFLOPS = 157.3    # MI355X fp32 dense matrix (and vector) peak, published
KERNEL_SLOTS = ["sample_gather", "grad", "apply"]


def measured_traffic_bytes(workload: str, kernel: str):
    """HBM bytes of one launch of `kernel` on `workload` as rocprofv3's FETCH_SIZE / WRITE_SIZE counters measured
    them (profiles/hbm_traffic.txt, which also says how); None where that kernel on that workload was not measured."""
    try:
        with open(TRAFFIC_TABLE) as f:
            for line in f:
                cols = line.split()
                if len(cols) >= 7 and not line.startswith("#") and cols[0] == workload and cols[1] == kernel:
                    return float(cols[6]) * 1e6
    except OSError:
        pass
    return None


def algorithmic_bytes_per_sample(w) -> int:
    """COO record (N indices + value) + one read and one write of every gathered factor row."""
    return 4 * (w.order + 1) + 8 * sum(w.J)


def algorithmic_flops_per_sample(w) -> int:
    """projections, GS and the core-gradient outer products: 2 flop per multiply-add each."""
    return 6 * sum(j * w.R for j in w.J)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # 1000 steps are ~0.13 s of GPU time on C2 (about 1 s on C3): long enough for steady state, the first
    # launches after a synchronisation run into an empty queue and a GPU that has clocked down
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="C2", choices=["C1", "C2", "C3", "C4", "C5", "O5", "O6", "O7", "O8", "O9", "O10"],
                    help="C2 is the headline workload; O5..O10 are the paper's order-scalability sweep")
    ap.add_argument("--kernel", default="auto")
    ap.add_argument("--sampling", default="entries", choices=["entries", "tiles"],
                    help="rule Psi is drawn by; 'tiles' is the library's variant rule (not the headline metric)")
    ap.add_argument("--layout", default="padded", choices=["padded", "exact"],
                    help="'exact' keeps rows at J_n floats (ftk_create flag FTK_LAYOUT_EXACT); by default ranks up to 16 "
                         "are held padded to 16 for orders 2..5.  No effect on C2 (J = R = 16).")
    ap.add_argument("--mode", default="sync", choices=["sync", "hogwild", "modewise"],
                    help="'hogwild' / 'modewise' time the in-place modes (not the headline metric)")
    ap.add_argument("--cpu-seconds", type=float, default=20.0, help="target wall time of the CPU-oracle leg (0: skip)")
    ap.add_argument("--spin-up-seconds", type=float, default=0.3,
                    help="untimed steps run before the W warm-up steps until this much wall time has passed, so that a "
                         "short run (K = 20) is not timed on a GPU that is still clocking up; 0: none")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus %d is not supported."
              % args.gpus, file=sys.stderr)
        return 2

    import torch
    from paper_2204_07104_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback.", file=sys.stderr)
        return 3

    w = synth.WORKLOADS[args.workload]
    t0 = time.time()
    idx, vals = synth.make_tensor(w)
    t_gen = time.time() - t0
    print("[bench] %s generated in %.1f s (nnz=%d)" % (w.name, t_gen, w.nnz), file=sys.stderr, flush=True)

    stream = torch.cuda.Stream()
    ft = binding.FastTucker(w.dims, idx, vals, w.J, w.R, w.init_seed,
                            flags=binding.FTK_LAYOUT_EXACT if args.layout == "exact" else 0)
    ft.ftk_set_stream(stream.cuda_stream)
    if args.kernel != "auto":
        ft.ftk_set_kernel(args.kernel)
    if args.sampling == "tiles":
        ft.ftk_set_sampling(binding.FTK_SAMPLE_TILES)
    if args.mode == "hogwild":
        ft.ftk_set_mode(binding.FTK_HOGWILD)
    elif args.mode == "modewise":
        ft.ftk_set_mode(binding.FTK_HOGWILD_MODEWISE)
    kernel_label = ft.ftk_kernel_name()
    if args.mode == "modewise":
        kernel_label = "%s, factor phase + core phase" % kernel_label
    print("[bench] context ready, gradient kernel = %s" % kernel_label, file=sys.stderr, flush=True)

    def run_steps(first: int, count: int) -> None:
        for t in range(first, first + count):
            ft.ftk_sample(w.sample_seed0 + t, w.n_samples)
            ft.ftk_sgd_step(w.lr_A, w.lr_B, w.lambda_A, w.lambda_B)

    K, W = args.steps, args.warmup
    # spin-up (untimed, before the warm-up steps): the first milliseconds after an idle period run at reduced clocks
    spun = 0
    t_spin = time.perf_counter()
    while time.perf_counter() - t_spin < args.spin_up_seconds:
        run_steps(spun, 50)
        torch.cuda.synchronize()
        spun += 50
    run_steps(spun, W)
    W += spun          # step numbers (sampling seeds) of the timed steps follow on
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    ev0.record(stream)
    run_steps(W, K)
    ev1.record(stream)
    torch.cuda.synchronize()
    ms_per_step = ev0.elapsed_time(ev1) / K
    value = w.n_samples / (ms_per_step * 1e-3)

    # second timed pass with per-kernel events
    ft.ftk_set_timing(True)
    run_steps(W + K, K)
    per_kernel = {}
    for slot, name in enumerate(KERNEL_SLOTS):
        ms, cnt = ft.ftk_get_timing(slot)
        per_kernel[name] = {"avg_ms": ms / max(cnt, 1), "launches": cnt, "ms_per_step": ms / K}
    ft.ftk_set_timing(False)
    rmse_after = ft.ftk_rmse()
    # the kernel's time per pass over Psi: its average launch (the two-phase mode launches it twice per step, and the
    # roofline is then held against both launches together)
    dominant = max(per_kernel, key=lambda k: per_kernel[k]["ms_per_step"])
    dom_ms = per_kernel[dominant]["ms_per_step"]
    bytes_per_launch = algorithmic_bytes_per_sample(w) * w.n_samples
    flops_per_launch = algorithmic_flops_per_sample(w) * w.n_samples
    achieved_gbs = bytes_per_launch / (dom_ms * 1e-3) / 1e9
    achieved_tflops = flops_per_launch / (dom_ms * 1e-3) / 1e12
    # the bound is whichever of the two lower limits on the launch time is the larger: moving the
    # algorithmic bytes at the HBM peak, or doing the three contractions at the fp32 matrix-core peak
    if flops_per_launch / (FP32_MFMA_PEAK_TFLOPS * 1e12) > bytes_per_launch / (HBM_PEAK_GBS * 1e9):
        head = {"bound": "mfma", "achieved": achieved_tflops, "peak": FP32_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved_tflops / FP32_MFMA_PEAK_TFLOPS}
    else:
        head = {"bound": "hbm", "achieved": achieved_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved_gbs / HBM_PEAK_GBS}
    # `traffic` only where this very kernel was measured on this workload under the default sampling rule and mode
    traffic = None
    if args.sampling == "entries" and args.mode == "sync" and args.layout == "padded":
        traffic = measured_traffic_bytes(w.name, dominant + ":" + kernel_label)
    roofline = {
        **head, "kernel": dominant + ":" + kernel_label,
        "traffic": traffic,
        # two different things, named apart: algorithmic bytes over time ("effective"), and the bytes the
        # HBM counters saw over the same time ("measured"; below the effective figure where rows hit in cache)
        "effective_gbs": achieved_gbs, "effective_frac": achieved_gbs / HBM_PEAK_GBS,
        "measured_hbm_gbs": None if traffic is None else traffic / (dom_ms * 1e-3) / 1e9,
        "measured_hbm_frac": None if traffic is None else traffic / (dom_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "bytes_per_sample": algorithmic_bytes_per_sample(w), "avg_kernel_ms": dom_ms,
        "whole_step_effective_gbs": bytes_per_launch / (ms_per_step * 1e-3) / 1e9,
        "whole_step_effective_frac": bytes_per_launch / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "flops_per_sample": algorithmic_flops_per_sample(w), "fp32_tflops_in_kernel": achieved_tflops,
        "per_kernel_ms": {k: v["avg_ms"] for k, v in per_kernel.items()},
        "launches_per_step": {k: v["launches"] / K for k, v in per_kernel.items()},
    }
    ft.close()
    if args.calibrate_copy:
        src = torch.ones(1 << 26, dtype=torch.float32, device="cuda")     # 256 MiB read, 256 MiB written
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cpu_baseline = None
    if args.cpu_seconds > 0:
        import oracle
        A, B = oracle.init_factors(w.init_seed, w.dims, w.J, w.R)
        probe = min(w.n_samples, 20_000)
        pos = oracle.sample_positions(w.sample_seed0, w.n_samples, w.nnz)
        t0 = time.perf_counter()
        oracle.sgd_step_sync(w.dims, idx, vals, [a.copy() for a in A], [b.copy() for b in B], pos[:probe],
                             w.lr_A, w.lr_B, w.lambda_A, w.lambda_B)
        rate = probe / max(time.perf_counter() - t0, 1e-9)
        per_step = min(w.n_samples, max(probe, int(rate * args.cpu_seconds)))
        n_cpu_steps = max(1, min(10, int(rate * args.cpu_seconds / per_step)))
        done = 0
        t0 = time.perf_counter()
        for t in range(n_cpu_steps):
            pos = oracle.sample_positions(w.sample_seed0 + t, w.n_samples, w.nnz)[:per_step]
            oracle.sgd_step_sync(w.dims, idx, vals, A, B, pos, w.lr_A, w.lr_B, w.lambda_A, w.lambda_B)
            done += per_step
        dt = time.perf_counter() - t0
        cpu_baseline = {
            "value": done / dt, "unit": "nonzeros/s", "cores": 1, "kind": "oracle",
            "sample": "%d step(s) of %d sampled nonzeros each on %s (same Psi seeds, sampling + step timed, %.1f s)"
                      % (n_cpu_steps, per_step, w.name, dt),
            "host_cpus": os.cpu_count(),
        }

    out = {
        "metric": "sampled nonzeros/sec per SGD step (order-%d %s nnz, %s); achieved HBM GB/s"
                  % (w.order, ("%dM" % (w.nnz // 1_000_000)) if w.nnz >= 1_000_000 else str(w.nnz),
                     ("J=R=%d" % w.R) if set(w.J) == {w.R} else
                     ("J=%s R=%d" % (w.J[0] if len(set(w.J)) == 1 else list(w.J), w.R))),
        "value": value, "unit": "nonzeros/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "spin_up_steps": spun,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: order-%d COO %s, nnz=%d, J=%s, R=%d, |Psi|=%d per step, %s step%s"
                               % (w.name, w.order, "x".join(str(d) for d in w.dims), w.nnz, list(w.J), w.R, w.n_samples,
                                  {"sync": "synchronous", "hogwild": "in-place (Hogwild)",
                                   "modewise": "in-place, mode by mode (Algorithm 1 as printed)"}[args.mode],
                                  "" if args.sampling == "entries" else ", tile-sampling variant"),
                   "kernel": roofline["kernel"], "rmse_after": rmse_after, "datagen_s": round(t_gen, 1)},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
