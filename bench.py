#!/usr/bin/env python3
"""Benchmark of the ExactOBS / OBQ hot path on one MI355X.

One "step" is one pass of the whole path over one synthetic layer that is already resident in
HBM: obc_hessian -> obc_invert -> (grid) -> per-row greedy solver -> (global step + gather for
unstructured pruning).  Prints ONE JSON line: whole-path row-steps/s, the roofline of the
dominant kernel measured with events on the library's stream, the same figures for the second
layer the performance target names (768 x 3072), and the CPU oracle timed on a bounded sample of
the headline workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--strategy auto|rank1|blocked]
    python bench.py --membench        # the plain read / write / copy kernels' GB/s instead
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# workload -> (layer, task)
WORKLOADS = {
    "conv256x2304-obq4": ("conv256x2304", "obq4"),
    "ffn768x3072-prune50": ("ffn768x3072", "prune50"),
    "ffn768x3072-obq4": ("ffn768x3072", "obq4"),
    "conv64x576-prune60": ("conv64x576", "prune60"),
    "conv64x576-nm24": ("conv64x576", "nm24"),
    "attn768x768-prune50": ("attn768x768", "prune50"),
    "attn768x768-obq4": ("attn768x768", "obq4"),
    "ffn3072x768-prune50": ("ffn3072x768", "prune50"),
    "ffn3072x768-obq4": ("ffn3072x768", "obq4"),
    "conv512x4608-prune50": ("conv512x4608", "prune50"),
    "conv512x4608-compound": ("conv512x4608", "compound50"),   # prune to 50 %, then OBQ 4-bit on survivors
    "lin16x32-prune50": ("lin16x32", "prune50"),
    # widened rows: block pruning (blocks of 4) to 50 % with the global step over the block traces, and
    # the sequential variant (inputs from a perturbed "compressed" model: re-fit, then OBQ)
    "conv256x2304-block4-50": ("conv256x2304", "block50"),
    "ffn768x3072-block4-50": ("ffn768x3072", "block50"),
    "conv256x2304-seqobq4": ("conv256x2304", "seqobq4"),
}
DEFAULT_WORKLOAD = "conv256x2304-obq4"
SECOND_WORKLOAD = "ffn768x3072-prune50"     # the other layer the target quotes its roofline figure on
HBM_PEAK_GBS = 8000.0
MFMA_F32_PEAK_TFLOPS = 157.3
# fp32 vector peak of the code as it is compiled here: 256 compute units x 4 SIMDs x 16 lanes x 2 flop
# (one FMA) x 2.4 GHz = 78.6 TFLOP/s.  The published 157.3 TFLOP/s counts two FMAs per lane and clock,
# which only the packed fp32 instructions reach; the library is built with them switched off.
VALU_F32_PEAK_TFLOPS = 256 * 4 * 16 * 2 * 2.4e9 / 1e12
BC = 4                                      # block size of the block-pruning workloads
NAMES = {"flush": "flush_kernel", "panel": "panel_kernel", "rank1": "rows_rank1_kernel"}


def run_workload(ctx, pkg, workload, steps, warmup, strategy, recover="auto"):
    """Time `steps` passes of the whole path on one layer; returns the figures and what the oracle leg needs."""
    import numpy as np
    import torch

    import obc_inputs

    layer, task = WORKLOADS[workload]
    W, X, spec = obc_inputs.make_layer(layer, device="cuda:0")
    R, d = W.shape
    N = X.shape[1]
    if task.startswith("block"):
        sparsity = int(task[-2:]) / 100.0
        k_steps, nm = d // BC, (0, 0)      # block steps per row
    elif task.startswith("prune") or task.startswith("compound"):
        sparsity = int(task[-2:]) / 100.0
        k_steps, nm = d, (0, 0)
    elif task == "nm24":
        k_steps, nm = d // 2, (2, 4)
    else:
        k_steps, nm = d, (0, 0)
    row_steps = R * k_steps * (BC if task.startswith("block") else 1)   # single eliminations
    if task.startswith("compound"):
        row_steps += R * d      # second pass: eliminations of the pruned + OBQ steps of the survivors

    # outputs allocated once (device memory is the caller's business, outside the timed path)
    H = torch.empty(d, d, device="cuda")
    out = dict(order=torch.empty(R, k_steps, dtype=torch.int32, device="cuda"),
               loss=torch.empty(R, k_steps, device="cuda"),
               W=torch.empty(R, d, device="cuda"))
    if task.endswith("obq4"):
        out["codes"] = torch.empty(R, d, dtype=torch.int32, device="cuda")
    Wfit = None
    if task == "seqobq4":
        # stand-in for the inputs of the already compressed model: the dense inputs, perturbed;
        # Y = the dense layer's outputs on the dense inputs
        torch.manual_seed(11)
        Y = (W @ X).contiguous()
        X = (X + 0.1 * X.std() * torch.randn_like(X)).contiguous()
        Cm = torch.empty(R, d, device="cuda")
        Wfit = torch.empty(R, d, device="cuda")
    qout = None
    if task.startswith("compound"):
        qout = dict(order=torch.empty(R, d, dtype=torch.int32, device="cuda"), loss=torch.empty(R, d, device="cuda"),
                    W=torch.empty(R, d, device="cuda"), codes=torch.empty(R, d, dtype=torch.int32, device="cuda"))
    want_trace = task.startswith("prune") or task.startswith("compound") or task.startswith("block")
    trace_bytes = R * k_steps * d * 4
    if want_trace and (trace_bytes > 120e9 or recover in ("closed", "replay")):
        want_trace = False        # largest layers (or on request): recover without the HBM trace
    if want_trace:
        out["trace"] = torch.empty(R, k_steps, d, device="cuda")
    ctx.workspace(max(ctx.rows_workspace_bytes(R, d, strategy), 1 << 20))

    ev = lambda: torch.cuda.Event(enable_timing=True)
    stage_ms = {"hessian": [], "invert": [], "rows": [], "global": []}
    grid = {}

    def one_step(record):
        e = [ev() for _ in range(5)]
        e[0].record()
        ctx.obc_hessian(X, damp_rel=0.01, H=H)
        e[1].record()
        if task == "seqobq4":
            ctx.obc_cross(X, Y, C=Cm)
            ctx.obc_refit(H, Cm, invert_in_place=True, W_out=Wfit)
        else:
            ctx.obc_invert(H)
        e[2].record()
        if task == "seqobq4":
            delta, offset, maxq = ctx.obc_minmax_grid(Wfit, 4)
            grid.update(delta=delta, offset=offset, maxq=maxq)
            res = ctx.obc_quant_rows(Wfit, H, delta, offset, maxq, strategy=strategy, out=out)
        elif task.startswith("block"):
            res = ctx.obc_prune_blocks(W, H, BC, want_trace=want_trace, strategy=strategy)
        elif task.startswith("obq"):
            delta, offset, maxq = ctx.obc_minmax_grid(W, 4)
            grid.update(delta=delta, offset=offset, maxq=maxq)
            res = ctx.obc_quant_rows(W, H, delta, offset, maxq, strategy=strategy, out=out)
        else:
            res = ctx.obc_prune_rows(W, H, k_steps=k_steps, nm=nm, want_trace=want_trace,
                                     strategy=strategy, out=out)
        e[3].record()
        result = res["W"]
        if task.startswith("block"):
            k = obc_inputs.target_count(sparsity, R, d) // BC
            counts, mask = ctx.obc_global_select(res["loss"], res["order"], k)
            result = ctx.obc_gather_trace(W, res["trace"], counts)
            out["order"] = res["order"]
            out["loss"] = res["loss"]
        elif task.startswith("prune") or task.startswith("compound"):
            k = obc_inputs.target_count(sparsity, R, d)
            counts, mask = ctx.obc_global_select(res["loss"], res["order"], k)
            if want_trace:
                result = ctx.obc_gather_trace(W, res["trace"], counts)
            elif recover == "closed":
                # group-OBS closed form on the mask; the largest per-row count sizes its workspace
                result = ctx.obc_reconstruct_rows(W, H, mask, max_pruned=int(counts.max()))
            else:
                result = ctx.obc_prune_rows(W, H, k_steps=k_steps, stop_counts=counts, strategy=strategy)["W"]
            if task.startswith("compound"):
                live = 1 - mask
                delta, offset, maxq = ctx.obc_minmax_grid(result, 4, live=live)
                result = ctx.obc_quant_rows(result, H, delta, offset, maxq, live=live, strategy=strategy, out=qout)["W"]
        e[4].record()
        if record:
            torch.cuda.synchronize()
            for name, a, b in (("hessian", 0, 1), ("invert", 1, 2), ("rows", 2, 3), ("global", 3, 4)):
                stage_ms[name].append(e[a].elapsed_time(e[b]))
        return result

    for _ in range(warmup):
        one_step(False)
    ctx.obc_check()
    torch.cuda.synchronize()
    ctx.obc_profile_begin()       # events around every row-solver launch, on the library's stream
    t0 = time.perf_counter()
    for _ in range(steps):
        one_step(True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kstats = ctx.obc_profile_end()
    ctx.obc_check()

    # ---- roofline of the dominant kernel of the row solver, from the events the library recorded
    # around each of its launches during the timed steps.  Algorithmic bytes / flops per launch are
    # those of the schedule the kernel implements (see include/obc.h, obc_profile_end).
    rows_s = 1e-3 * float(np.mean(stage_ms["rows"]))
    if task.startswith("compound"):      # the second row-solver pass (OBQ on the survivors) sits in the last stage
        rows_s += 1e-3 * float(np.mean(stage_ms["global"]))
    kern = {k: v for k, v in kstats.items() if v["launches"] > 0}
    dom = max(kern, key=lambda k: kern[k]["ms"])
    ds = kern[dom]
    gbs = ds["bytes"] / (1e-3 * ds["ms"]) / 1e9 if ds["ms"] > 0 else 0.0
    tfs = ds["flops"] / (1e-3 * ds["ms"]) / 1e12 if ds["ms"] > 0 else 0.0
    if dom == "rank1" and ds["bytes"] == 0:      # LDS-resident: bounded by the fp32 vector units
        roofline = {"bound": "alu", "kernel": NAMES[dom], "achieved": tfs, "peak": VALU_F32_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": tfs / VALU_F32_PEAK_TFLOPS, "traffic": None}
    else:
        roofline = {"bound": "hbm", "kernel": NAMES[dom], "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": gbs / HBM_PEAK_GBS, "traffic": None}
    # measured HBM bytes per launch of the dominant kernel, from the stored rocprofv3 counter runs of
    # this same command (profiles/hbm_traffic_<workload>.txt), when such a summary exists
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_%s.txt" % workload.replace("-", "_"))
    if os.path.exists(tpath) and strategy == pkg.STRATEGY_AUTO:
        for ln in open(tpath):
            if ln.startswith("family %s " % NAMES[dom]):
                roofline["traffic"] = float(ln.split("traffic_bytes_per_launch=")[1].split()[0])
    # the row solver as a whole: the algorithmic bytes of all its launches (panels and flushes, the
    # schedule they implement) over the time of the whole rows call; and, for context, the bytes the
    # literal Algorithm 1 would move (read + write the whole d x d matrix every step: 8 d^2 per
    # row-step) over the same time -- an equivalent rate, far above the peak because the blocked,
    # symmetric, shrinking schedule moves that many fewer bytes
    solver_bytes = sum(v["bytes"] for v in kern.values()) / steps
    literal_bytes = 8.0 * d * d * float(row_steps)
    roofline.update({
        "launches_per_step": ds["launches"] / steps, "avg_launch_ms": ds["ms"] / ds["launches"],
        "alg_bytes_per_launch": ds["bytes"] / ds["launches"], "mfma_tflops": tfs,
        "mfma_frac": tfs / MFMA_F32_PEAK_TFLOPS,
        "share_of_rows_time": ds["ms"] / steps / (1e3 * rows_s),
        "row_steps_per_s_rows_call": row_steps / rows_s,
        "solver": {"alg_bytes_per_step": solver_bytes, "rows_call_ms": 1e3 * rows_s,
                   "GB/s": solver_bytes / rows_s / 1e9, "frac": solver_bytes / rows_s / 1e9 / HBM_PEAK_GBS},
        "literal_S": {"bytes_per_step": literal_bytes, "equiv_GB/s": literal_bytes / rows_s / 1e9,
                      "equiv_frac": literal_bytes / rows_s / 1e9 / HBM_PEAK_GBS},
        "kernels": {NAMES[k]: {"launches_per_step": v["launches"] / steps, "ms_per_step": v["ms"] / steps,
                               "GB/s": v["bytes"] / (1e-3 * v["ms"]) / 1e9, "TFLOP/s": v["flops"] / (1e-3 * v["ms"]) / 1e12}
                    for k, v in kern.items()},
    })
    hess_tf = float(d) * d * N / (1e-3 * float(np.mean(stage_ms["hessian"]))) / 1e12   # useful flops: one triangle
    return dict(workload=workload, task=task, R=R, d=d, N=N, k_steps=k_steps, nm=nm, row_steps=row_steps,
                ms_per_step=1e3 * wall / steps, value=row_steps / (wall / steps),
                stages_ms={k: float(np.mean(v)) for k, v in stage_ms.items() if v}, roofline=roofline,
                hessian_mfma_frac=hess_tf / MFMA_F32_PEAK_TFLOPS,
                W=(Wfit if task == "seqobq4" else W), Hinv=H, out=out, grid=grid)


def oracle_leg(r, cpu_rows):
    """The oracle on the host cores over a bounded sample of rows, fed what the GPU solver was fed
    (its fp32 inverse Hessian, weights and grid), and the agreement of the two on those rows."""
    import numpy as np

    from oracle import oracle as orc

    task, R, d, k_steps, nm = r["task"], r["R"], r["d"], r["k_steps"], r["nm"]
    block = task.startswith("block")
    threads = min(os.cpu_count() or 1, 16)
    # keep the sample to roughly 10-30 s: the oracle costs ~ k d^2 / 3 inner iterations per row
    per_row_s = (k_steps * (BC if block else 1) * d * d / 3.0) / 0.7e9
    n_rows = cpu_rows or threads * max(1, int(round(15.0 / max(per_row_s, 1e-9))))
    n_rows = min(n_rows, R)
    while n_rows > threads and per_row_s * n_rows / threads > 30:
        n_rows //= 2
    A64 = r["Hinv"].cpu().numpy().astype(np.float64)
    Wn = r["W"][:n_rows].cpu().numpy().astype(np.float64)
    quant = task.endswith("obq4")
    if quant:
        dl = r["grid"]["delta"][:n_rows].cpu().numpy().astype(np.float64)
        of = r["grid"]["offset"][:n_rows].cpu().numpy().astype(np.float64)
        maxq = r["grid"]["maxq"]
    t1 = time.perf_counter()
    if block:
        ro = orc.block_prune_rows(A64, Wn, BC, n_threads=threads)
    elif quant:
        ro = orc.quant_rows(A64, Wn, dl, of, maxq, n_threads=threads)
    else:
        ro = orc.prune_rows(A64, Wn, k_steps=k_steps, nm=nm, n_threads=threads)
    cpu_s = time.perf_counter() - t1
    base = {
        "value": n_rows * k_steps * (BC if block else 1) / cpu_s, "unit": "row-steps/s", "cores": int(ro["threads"]),
        "kind": "oracle", "sample": "%d of %d rows of %s, all %d steps each, %.1f s" % (
            n_rows, R, r["workload"], k_steps, cpu_s),
    }
    # Agreement of the timed GPU result with the oracle on the sampled rows (outside the timed
    # part).  Orders are compared entry by entry; a row whose order differs is replayed by the
    # oracle along the GPU's order, and every GPU pick must then score within 1e-6 relative of the
    # oracle's minimum at that step (two near-tied picks taken in the other order give the same
    # state two steps later).
    g_order = r["out"]["order"][:n_rows].cpu().numpy()
    same = g_order == ro["order"]
    agree = {"order_entries_equal": float(np.mean(same)), "rows_with_swaps": 0, "near_ties": 0, "beyond_gap": 0}
    bad_rows = [i for i in range(n_rows) if not same[i].all()]
    agree["rows_with_swaps"] = len(bad_rows)
    for i in bad_rows[:8]:                       # bounded: each replay is one more oracle row
        f = g_order[i].astype(np.int32)
        if block:
            rr = orc.block_prune_row(A64, Wn[i], BC, forced=f)
        elif quant:
            rr = orc.quant_row(A64, Wn[i], (float(dl[i]), float(of[i]), maxq), forced=f)
        else:
            rr = orc.prune_row(A64, Wn[i], k_steps=k_steps, nm=nm, forced=f)
        gap = rr.pick_score - rr.min_score
        tol = 1e-6 * rr.min_score + 1e-12 * float(np.max(rr.min_score))
        agree["near_ties"] += int(np.count_nonzero((gap > 0) & (gap <= tol)))
        agree["beyond_gap"] += int(np.count_nonzero(gap > tol))
    agree["rows_replayed"] = min(len(bad_rows), 8)
    base["agreement"] = agree
    return base


def membench(ctx):
    """GB/s of the library's plain read / write / copy kernels over 4 GiB buffers."""
    import torch

    nbytes = 4 << 30
    src = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    res = {"bytes_per_buffer": nbytes}
    for name, kind, streaming, moved in (("read", 0, False, nbytes), ("write", 1, False, nbytes),
                                         ("write_streaming", 1, True, nbytes), ("copy", 2, False, 2 * nbytes),
                                         ("copy_streaming", 2, True, 2 * nbytes)):
        ms = ctx.obc_membench(kind, src, dst, nbytes, reps=5, streaming=streaming)
        res[name] = {"ms": ms, "GB/s": moved / (1e-3 * ms) / 1e9, "frac_of_peak": moved / (1e-3 * ms) / 1e9 / HBM_PEAK_GBS}
    # the matrix cores on a loop of independent MFMA instructions (data-sheet: 157.3 / 78.6 TFLOP/s)
    mfma = {"f32_32x32x2_TFLOP/s": ctx.obc_mfmabench(0), "f64_16x16x4_TFLOP/s": ctx.obc_mfmabench(1),
            "f32_peak": MFMA_F32_PEAK_TFLOPS, "f64_peak": 78.6}
    print(json.dumps({"membench": res, "peak_GB/s": HBM_PEAK_GBS, "mfmabench": mfma}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD, choices=sorted(WORKLOADS))
    ap.add_argument("--strategy", default="auto", choices=["auto", "rank1", "blocked"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-second-layer", action="store_true",
                    help="skip the 768 x 3072 layer that the default run times after the headline workload")
    ap.add_argument("--cpu-rows", type=int, default=0, help="rows in the oracle sample (0 = one per host thread)")
    ap.add_argument("--recover", default="auto", choices=["auto", "trace", "closed", "replay"],
                    help="pruning workloads: how the weights of the global step's mask are recovered (auto: from the "
                         "HBM trace when it fits, else by replay; closed: the group-OBS closed form)")
    ap.add_argument("--membench", action="store_true", help="time the plain read / write / copy kernels and exit")
    ap.add_argument("--calib-copy", action="store_true",
                    help="after the timed region run one plain 1 GiB device copy (calibrates rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters against a kernel of known traffic)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the row solver shards trivially over rows, "
                 "but no multi-GPU path exists here); run with --gpus 1")

    import torch

    import paper_2208_11580_amd as pkg

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    ctx = pkg.Context()
    if args.membench:
        membench(ctx)
        return
    strategy = {"auto": pkg.STRATEGY_AUTO, "rank1": pkg.STRATEGY_RANK1, "blocked": pkg.STRATEGY_BLOCKED}[args.strategy]
    r = run_workload(ctx, pkg, args.workload, args.steps, args.warmup, strategy, args.recover)
    if args.calib_copy:
        nb = 1 << 30                                   # 1 GiB read, 1 GiB written
        src = torch.zeros(nb, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        ctx.obc_membench(2, src, dst, nb, reps=1)      # (one warm-up + one timed launch of the copy kernel)
        del src, dst

    line = {
        "metric": "ExactOBS row-steps/sec per layer + % fp32 VALU/HBM roofline, 1 MI355X",
        "value": r["value"], "unit": "row-steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "d_row": r["R"], "d_col": r["d"], "n_samples": r["N"], "task": r["task"],
                   "strategy": args.strategy, "row_steps": r["row_steps"], "recover": args.recover},
        "stages_ms": r["stages_ms"],
        "hessian_mfma_frac": r["hessian_mfma_frac"],
        "roofline": r["roofline"],
    }
    # ---- the oracle on the host cores, on a bounded sample of rows of the same layer
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = oracle_leg(r, args.cpu_rows)
    # ---- the second layer of the target, same path, after the headline workload's buffers are gone
    if args.workload == DEFAULT_WORKLOAD and args.strategy == "auto" and not args.no_second_layer:
        del r
        ctx.release_workspace()
        torch.cuda.empty_cache()
        s = run_workload(ctx, pkg, SECOND_WORKLOAD, min(args.steps, 3), min(args.warmup, 1), strategy)
        line["second_layer"] = {
            "workload": SECOND_WORKLOAD, "d_row": s["R"], "d_col": s["d"], "n_samples": s["N"],
            "value": s["value"], "unit": "row-steps/s", "ms_per_step": s["ms_per_step"], "steps": min(args.steps, 3),
            "stages_ms": s["stages_ms"], "hessian_mfma_frac": s["hessian_mfma_frac"], "roofline": s["roofline"],
        }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
