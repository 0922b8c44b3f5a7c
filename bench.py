#!/usr/bin/env python3
"""Benchmark of the CCE- hot path on one MI355X: forward + backward of the loss over one synthetic batch.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 5] [--algo auto|gather|tile]

A step is one cce_neg_forward followed by one cce_neg_backward on inputs already resident in HBM.  The line printed on
stdout is one JSON object: whole-job positions/s of the headline workload (the largest single-GPU one, c5, unless
--config names another), the roofline of its dominant kernel (timed with events on the launch stream), the fp64 CPU
oracle timed on a bounded sample of the same workload, and, under "other_workloads", the same step measured on the
remaining workloads (c1: microseconds only; c2-c4: step time, positions/s, dominant kernel and its roofline fraction).
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_BF16_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak
EXP_PER_S = 12.5e12           # measured v_exp_f32 rate of the whole chip (profiles/microbenchmarks.md)
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E peak
PEAK_F32_VALU_TFLOPS = 157.3


def algorithmic_work(w):
    """Algorithmic flops and minimum HBM bytes of one forward+backward, counted on valid positions only.

    flops: four GEMM-equivalents (scores forward, scores recomputed, dH, dE), 2 flop per multiply-add:
           8 * n_cand * d per valid position, n_cand = K+1 (or V for the full catalogue).
    bytes: every operand the method must move once: H read in both passes, the gathered candidate rows in both passes,
           dH written, dE rows written once (write-once accounting), ids, per-position vectors.
    """
    nv = w.n_valid
    esz = 4 if w.in_dtype == "f32" else 2
    n_cand = w.V if w.neg_mode == 2 else w.K + 1
    flops = 8.0 * n_cand * w.d * nv
    row = w.d * esz
    if w.neg_mode == 1:      # per-position: every candidate row is fetched per position, twice; dE rows written once each
        gathered = 2.0 * nv * n_cand * row
        dE_bytes = float(nv) * n_cand * w.d * 4
        ids = 2.0 * nv * w.K * 4
    else:                    # shared / full: the candidate block is read once per pass, target rows per position
        n_neg_rows = w.V if w.neg_mode == 2 else w.K
        gathered = 2.0 * (n_neg_rows * row + (nv * row if w.neg_mode == 0 else 0))
        dE_bytes = float(n_neg_rows) * w.d * 4 + (float(nv) * w.d * 4 if w.neg_mode == 0 else 0)
        ids = 2.0 * (w.K * 4 if w.neg_mode == 0 else 0)
    per_pos = nv * (2 * row + w.d * 4) + w.N * (4 + 1 + 4 * 4)   # H twice, dH fp32, tgt, mask, loss/lse/lse/g
    return flops, gathered + dE_bytes + ids + per_pos


def kernel_work(w, family, fused=False):
    """Algorithmic work of ONE launch of a kernel family: ("mfma", flops) or ("hbm", bytes).

    Matrix-core kernels: 2 * n_cols * d flop per valid position and GEMM-equivalent, n_cols = K (V for the full
    catalogue).  A step has four of them (scores, scores recomputed in the backward pass as in Alg. 2, dH, dE), and each
    is counted in the launch that carries it out, once.  Separate passes: forward one (scores), dH pass two (scores
    recomputed, dH), dE pass one (dE; its own second recomputation of the scores is overhead and does not count);
    hidden sizes up to 128 run the dH and the dE pass in one launch (tile_bwd, three).  With fuse_dH the forward launch
    carries scores and dH (two), and the backward pass's one recomputation of the scores happens in the dE launch (two).
    Row-gather kernels: the candidate rows of every valid position (K+1 rows of d elements), the ids, H, and for the
    backward pass dH and every dE row written once.
    """
    nv = w.n_valid
    esz = 4 if w.in_dtype == "f32" else 2
    n_cols = w.V if w.neg_mode == 2 else w.K
    gemm = 2.0 * n_cols * w.d * nv
    if family == "tile_fwd":
        return "mfma", gemm
    if family in ("tile_dh", "tile_fdh"):   # scores + dH; the fused forward + dH pass (fuse_dH) is the same two
        return "mfma", 2 * gemm
    if family == "tile_de":
        return "mfma", (2 * gemm if fused else gemm)
    if family == "tile_bwd":   # dH and dE pass in one launch
        return "mfma", 3 * gemm
    if family == "dh_scale":   # U read, dH written (fp32 both), grad_loss
        return "hbm", float(nv) * (8 * w.d + 4) + w.N
    if family == "fdh_merge":  # partial rows read once, U written
        return "hbm", float(nv) * 8 * w.d
    if family == "bwd_pre":    # per valid position: H row, correct item's row, five scalars in, three out
        return "hbm", float(nv) * (2 * w.d * esz + 32)
    n_cand = w.V if w.neg_mode == 2 else w.K + 1
    rows = float(nv) * n_cand * w.d * esz
    ids = float(nv) * (w.K if w.neg_mode == 1 else 0) * 4
    if family == "gather_fwd":
        return "hbm", rows + ids + nv * w.d * esz + w.N * 13
    if family == "gather_bwd":
        if w.neg_mode == 1:  # per-position: dE leaves through the inverted-index pass, this kernel writes dH only
            return "hbm", rows + ids + nv * w.d * esz + nv * w.d * 4 + w.N * 13
        return "hbm", rows + ids + nv * w.d * esz + float(nv) * n_cand * w.d * 4 + nv * w.d * 4 + w.N * 13
    pairs = float(nv) * w.K
    if family == "item_de":
        # per (position, negative) pair: the position's H row and the pair's id; per touched table row: E read once,
        # dE read and written once.  Touched rows: expected number of distinct ids among nv*K uniform draws.
        touched = w.V * (1.0 - math.exp(-pairs / w.V))
        return "hbm", pairs * (w.d * esz + 4) + touched * (w.d * esz + 2 * w.d * 4)
    if family == "index":
        # inverted index: ids read by the counting and by the filing pass, (id, position) pairs written and read once
        # by each of the two sort levels, positions filed under their item
        return "hbm", pairs * (2 * 4 + 2 * 8 + 2 * 8 + 4)
    if family == "pos_scatter":
        return "hbm", float(nv) * (w.d * esz + 2 * w.d * 4 + 8)
    return "hbm", 0.0


def measured_traffic(workload, family):
    """HBM bytes per step of a kernel family, measured with rocprofv3 counters and kept under profiles/ (None when no
    record exists for this workload and family)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) >= 4 and not line.startswith("#") and f[0] == workload and f[1] == family:
            return float(f[2]) + float(f[3])
    return None


def measure(w, args, *, headline: bool) -> dict:
    """K timed steps of forward + backward on workload w, then the per-kernel breakdown.  Returns the result fields."""
    import numpy as np
    import torch

    import paper_2509_09682_amd as P
    from paper_2509_09682_amd.runner import to_device

    steps, warmup = (args.steps, args.warmup) if headline else (args.other_steps, args.warmup)
    H, E, tgt, neg, mask = to_device(w)
    algo = {"auto": P.CCE_ALGO_AUTO, "gather": P.CCE_ALGO_GATHER, "tile": P.CCE_ALGO_TILE}[args.algo]
    in_dt = P.CCE_F32 if w.in_dtype == "f32" else P.CCE_BF16
    filter_eps = args.filter_eps if headline else 0.0
    fuse = 0 if (args.no_fuse_dh or filter_eps > 0) else 1
    desc = P.make_desc(w.N, w.V, w.d, w.K, in_dt, w.neg_mode, mask_target_collisions=w.mask_collisions,
                       validate_indices=0, algo=algo, fuse_dH=fuse)
    # a training step runs the backward pass right after the forward pass of the same batch on the same workspace:
    # the backward call may then reuse what the forward call left there
    desc_bwd = P.make_desc(w.N, w.V, w.d, w.K, in_dt, w.neg_mode, mask_target_collisions=w.mask_collisions,
                           validate_indices=0, algo=algo, reuse_forward_prep=0 if args.no_reuse_prep else 1,
                           filter_eps=filter_eps, fuse_dH=fuse)
    ws = P.new_workspace(desc)
    loss = torch.empty(w.N, device="cuda")
    lse = torch.empty(w.N, device="cuda")
    g = torch.from_numpy(w.g).cuda()
    dH = torch.empty((w.N, w.d), device="cuda")
    dE = torch.zeros((w.V, w.d), device="cuda")

    smp = None
    sampler = args.sampler if headline else "none"
    if sampler != "none":
        from paper_2509_09682_amd.runner import device_sampler
        from workloads import alias_table, popularity_weights
        table = ()
        if sampler == "alias":   # the popularity law of workload c5 over a seeded rank -> id permutation
            table = alias_table(popularity_weights(np.random.default_rng(3).permutation(w.V).astype(np.int32), 1.2, 0.75))
        smp, smp_keep = device_sampler(P.CCE_SAMPLER_UNIFORM if sampler == "uniform" else P.CCE_SAMPLER_ALIAS,
                                       w.notes["seed"], 0, *table)
        neg = None
        step_no = [0]

    def forward():
        if smp is None:
            return P.cce_neg_forward(desc, H, E, tgt, neg, mask, loss, lse, ws)
        step_no[0] += 1
        smp.stream = step_no[0] & 0xFFFFFFFF     # other negatives every step; the backward call repeats the number
        return P.cce_neg_forward_sampled(desc, smp, H, E, tgt, mask, loss, lse, ws)

    def backward():
        if smp is None:
            return P.cce_neg_backward(desc_bwd, H, E, tgt, neg, mask, lse, g, dH, dE, ws)
        return P.cce_neg_backward_sampled(desc_bwd, smp, H, E, tgt, mask, lse, g, dH, dE, ws)

    def step():
        forward()
        backward()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()

    # timed region: exactly K steps bracketed by synchronisation, nothing else on the stream.  Peak memory of the
    # region: everything the step needs (inputs, outputs, workspace) is allocated by now and the steps allocate nothing.
    torch.cuda.reset_peak_memory_stats()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_step = (t1 - t0) * 1e3 / steps
    peak_allocated = int(torch.cuda.max_memory_allocated())
    free_b, total_b = torch.cuda.mem_get_info()          # hipMemGetInfo: the device's own view, allocator caches and
    device_in_use = int(total_b - free_b)                # the runtime's context included

    # forward / backward split of the same steps (events on the launch stream), outside the timed region
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    for k in range(steps):
        ev[k][0].record()
        forward()
        ev[k][1].record()
        backward()
        ev[k][2].record()
    torch.cuda.synchronize()
    fwd_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
    bwd_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in ev]))

    # cold caches: a 1 GiB write between steps evicts L2 and the Infinity Cache
    cold_ms = None
    if headline and args.cold_reps > 0:
        scratch = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
        c = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.cold_reps)]
        for k in range(args.cold_reps):
            scratch.fill_(float(k))
            c[k][0].record()
            step()
            c[k][1].record()
        torch.cuda.synchronize()
        cold_ms = float(np.median([e[0].elapsed_time(e[1]) for e in c]))
        del scratch

    # dE zero-fill, reported apart from the step (dE is an accumulate-into buffer owned by the caller)
    z0, z1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    z0.record()
    dE.zero_()
    z1.record()
    torch.cuda.synchronize()
    memset_ms = z0.elapsed_time(z1)

    # per-kernel durations: the same K steps once more with the library's event brackets switched on
    P.cce_neg_profile_enable(True)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    fam = P.cce_neg_profile_read()
    P.cce_neg_profile_enable(False)
    kernels = {k: {"avg_ms": ms / n, "launches_per_step": n / steps} for k, (ms, n) in fam.items()}
    # the dominant kernel family and its time per step (a family that launches several times per step, e.g. the item pass
    # of the sliced inverted index, is taken as a whole: its algorithmic work below is per step as well)
    dominant = max(fam, key=lambda k: fam[k][0])
    dom_ms = fam[dominant][0] / steps

    flops, bytes_min = algorithmic_work(w)
    bound, work = kernel_work(w, dominant, fused=bool(fuse))
    if bound == "mfma":
        peak = PEAK_MFMA_BF16_TFLOPS if w.in_dtype == "bf16" else PEAK_F32_VALU_TFLOPS
        roof = {"bound": "mfma", "kernel": dominant, "achieved": work / (dom_ms * 1e-3) / 1e12, "peak": peak,
                "unit": "TFLOP/s"}
    else:
        roof = {"bound": "hbm", "kernel": dominant, "achieved": work / (dom_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = measured_traffic(w.name, dominant)
    roof["avg_launch_ms"] = dom_ms
    roof["launches_per_step"] = fam[dominant][1] / steps
    roof["algorithmic_per_launch"] = work

    mfma_bound = w.in_dtype == "bf16" and w.neg_mode != 1
    whole = {"tflops": flops / (ms_step * 1e-3) / 1e12, "frac_mfma_peak": flops / (ms_step * 1e-3) / 1e12 / PEAK_MFMA_BF16_TFLOPS,
             "gbytes_per_s": bytes_min / (ms_step * 1e-3) / 1e9, "frac_hbm_peak": bytes_min / (ms_step * 1e-3) / 1e9 / PEAK_HBM_GBS,
             "bound": "mfma" if mfma_bound else "hbm"}
    whole["frac"] = whole["frac_mfma_peak"] if mfma_bound else whole["frac_hbm_peak"]
    config = {
        "workload": w.name, "N": w.N, "n_valid": w.n_valid, "d": w.d, "V": w.V, "K": w.K,
        "neg_mode": ["shared", "per_position", "full"][w.neg_mode], "algo": args.algo,
        "reuse_forward_prep": not args.no_reuse_prep, "fuse_dH": bool(fuse), "filter_eps": filter_eps, "sampler": sampler,
        "valid_positions_per_s": w.n_valid / (ms_step * 1e-3),
        "fwd_ms": fwd_ms, "bwd_ms": bwd_ms, "cold_ms_per_step": cold_ms, "dE_zero_fill_ms": memset_ms, "kernels": kernels,
        "exp_ceiling_ms": 2.0 * w.n_valid * ((w.V if w.neg_mode == 2 else w.K) + 1) / EXP_PER_S * 1e3,
        "algorithmic_gflop": flops / 1e9, "algorithmic_mbytes": bytes_min / 1e6,
        "whole_step": whole,
        "hbm_bytes": {"inputs": int(H.numel() * H.element_size() + E.numel() * E.element_size() + tgt.numel() * 4
                                    + (0 if neg is None else neg.numel() * 4) + w.N),
                      "outputs": int(w.N * 8 + dH.numel() * 4 + dE.numel() * 4),
                      "workspace": int(ws.numel()),
                      "peak_allocated_in_timed_region": peak_allocated,
                      "device_in_use_hipMemGetInfo": device_in_use},
    }
    return {"ms_per_step": ms_step, "value": w.N / (ms_step * 1e-3), "steps": steps, "config": config, "roofline": roof}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=5,
                    help="headline workload 1..5 (default 5: the largest single-GPU workload; the metric names no config)")
    ap.add_argument("--others", default="auto",
                    help="comma-separated workloads measured as well and reported under other_workloads "
                         "(auto: the remaining ones of 1..5 when the headline is the default, none otherwise)")
    ap.add_argument("--other-steps", type=int, default=30, help="timed steps per workload of --others")
    ap.add_argument("--algo", default="auto", choices=["auto", "gather", "tile"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cold-reps", type=int, default=5, help="steps timed with a 1 GiB cache-evicting write in front (0 = skip)")
    ap.add_argument("--filter-eps", type=float, default=0.0, help="gradient filtering threshold (full-catalogue workload c4 only)")
    ap.add_argument("--peaked", action="store_true", help="hidden states that point at their target row: a concentrated softmax, as late in training (c4)")
    ap.add_argument("--no-reuse-prep", action="store_true", help="backward recomputes what the forward call left in the workspace")
    ap.add_argument("--no-fuse-dh", action="store_true",
                    help="forward computes lse only and the backward call runs a dH pass of its own (five score-sized products "
                         "per step instead of four)")
    ap.add_argument("--sampler", default="none", choices=["none", "uniform", "alias"],
                    help="draw the negatives inside the kernels (shared / per-position workloads): no index array is read")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target oracle time for the cpu_baseline sample")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="BYTES",
                    help="only run five plain device copies of BYTES (reference for the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    if not torch.cuda.is_available():
        print("bench.py needs a GPU (no CPU fallback exists for the product path)", file=sys.stderr)
        return 2

    if args.copy_calibration:
        src = torch.empty(args.copy_calibration, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": args.copy_calibration, "copies": 5}))
        return 0

    from workloads import config

    w = config(args.config)
    if args.peaked:
        from workloads import bf16_bits_from_f32, f32_from_bf16_bits
        rng = np.random.default_rng(7)
        Ef = f32_from_bf16_bits(w.E)
        scale = 9.0 / float(np.mean(np.sum(Ef * Ef, axis=1)))   # correct-item score about 9 above the rest
        w.H = bf16_bits_from_f32((scale * Ef[w.tgt] + 0.5 * rng.standard_normal((w.N, w.d)).astype(np.float32)).astype(np.float32))
        w.name += "_peaked"
    res = measure(w, args, headline=True)

    out = {
        "metric": "CE- fwd+bwd positions/sec at 1 GPU",
        "value": res["value"],
        "unit": "positions/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if w.in_dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": res["config"],
        "roofline": res["roofline"],
    }

    if not args.no_cpu_baseline:
        from oracle import cce_oracle as O

        valid_idx = np.flatnonzero(w.mask)
        pilot = valid_idx[: min(64, valid_idx.size)].astype(np.int64)
        t = time.perf_counter()
        O.run_workload(w, sel=pilot, want_dE="compact")
        dt = max(time.perf_counter() - t, 1e-4)
        n_sample = int(min(valid_idx.size, max(64, args.cpu_seconds / (dt / pilot.size))))
        sample = valid_idx[:n_sample].astype(np.int64)
        t = time.perf_counter()
        O.run_workload(w, sel=sample, want_dE="compact")
        dt = time.perf_counter() - t
        # scale to the metric's unit: positions as passed (padded ones cost the oracle nothing)
        out["cpu_baseline"] = {
            "value": (n_sample / dt) * (w.N / max(w.n_valid, 1)), "unit": "positions/s", "cores": O.num_threads(),
            "kind": "oracle", "sample": f"first {n_sample} valid positions of {w.name} (fwd+bwd, fp64, {dt:.1f} s)",
        }

    # the remaining workloads, one after the other on the same GPU (inputs of the previous one are released first)
    if args.others == "auto":
        others = [i for i in (1, 2, 3, 4, 5) if i != args.config] if (args.config == 5 and not args.peaked) else []
    else:
        others = [int(x) for x in args.others.split(",") if x.strip()]
    del w
    out["other_workloads"] = []
    for idx in others:
        torch.cuda.empty_cache()
        wo = config(idx)
        r = measure(wo, args, headline=False)
        c, roof = r["config"], r["roofline"]
        entry = {"workload": wo.name, "ms_per_step": r["ms_per_step"], "us_per_step": r["ms_per_step"] * 1e3,
                 "steps": r["steps"]}
        if idx != 1:   # c1 is a correctness workload (30 MFLOP): latency only, no roofline claim
            entry.update({
                "positions_per_s": r["value"], "valid_positions_per_s": c["valid_positions_per_s"],
                "dominant_kernel": roof["kernel"], "bound": roof["bound"], "frac": roof["frac"],
                "achieved": roof["achieved"], "unit": roof["unit"], "traffic": roof["traffic"],
                "whole_step_bound": c["whole_step"]["bound"], "whole_step_frac": c["whole_step"]["frac"],
                "fwd_ms": c["fwd_ms"], "bwd_ms": c["bwd_ms"], "dE_zero_fill_ms": c["dE_zero_fill_ms"],
                "kernels": {k: round(v["avg_ms"], 5) for k, v in c["kernels"].items()},
                "peak_allocated_in_timed_region": c["hbm_bytes"]["peak_allocated_in_timed_region"],
            })
        out["other_workloads"].append(entry)
        del wo

    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
