#!/usr/bin/env python3
"""Benchmark of the local Newton-CG x-update hot path on one MI355X.

One step = one pass of the whole hot path over the image-like workload
(n = 60000, p = 784, C = 10, seeded synthetic data resident in HBM):
    100 Hessian-vector products (random V, cycling 4 pre-generated directions),
    100 objective+gradient evaluations,
    1 local Newton-CG solve (10 Newton iterations, 10 CG iterations each, Armijo line search).
The headline value is Hessian-vector products per second; the other rates are
reported in "extra".  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak, GB/s
HV_PER_STEP = 100
LG_PER_STEP = 100
# HBM bytes per nadmm_hessvec call from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised under
# profiles/ (scaled by a plain copy of known size); counters cannot be read inside a timing run.  Every entry
# names the summary it comes from and the digest of the kernel sources it was measured with: if the sources of
# that kernel path have changed since, the line reports traffic = null instead of a stale figure.
MEASURED_HV_TRAFFIC = {
    ("image_like_60000x784_C10", 2): (207.1e6, "profiles/hessvec_fused_image_like_60000x784_C10.md", "d910ee797784"),
    ("tall_binary_1375000x28_C2", 3): (154.4e6, "profiles/hessvec_thin_tall_binary_1375000x28_C2.md", "e5e4ee407ae4"),
    ("wide_50000x3072_C10", 4): (1259.6e6, "profiles/hessvec_sliced_wide_50000x3072_C10.md", "fc83e16f100a"),
    ("large_multiclass_250000x2000_C20", 4): (4220.8e6, "profiles/hessvec_sliced_large_multiclass_250000x2000_C20.md", "fc83e16f100a"),
    # sparse storage: bytes between the L2 caches and the memory side, most of them operand rows served by the Infinity Cache
    ("e18_like_40628x279998_C20_sparse", 5): (12480.0e6, "profiles/hessvec_sparse_e18_like_40628x279998_C20.md", "8090591d36f9"),
}
PATH_SOURCES = {1: ["nadmm_generic.hip", "nadmm_rows16.h"], 2: ["nadmm_fused.hip", "nadmm_cgstep.h"], 3: ["nadmm_thin.hip", "nadmm_cgstep.h"],
                4: ["nadmm_sliced.hip", "nadmm_rows16.h"], 5: ["nadmm_sparse.hip", "nadmm_generic.hip", "nadmm_rows16.h"]}
DTYPE = "f32 data and results; products on bf16 MFMA with split operands (3 terms, 6 for the logits A X), f32 accumulate; f64 scalar sums"


def source_digest(path):
    """Digest of the kernel sources of one kernel path (plus the shared helpers and the reduction)."""
    import hashlib
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_1807_07132_amd", "csrc")
    h = hashlib.sha256()
    for name in PATH_SOURCES[path] + ["nadmm_mfma.h", "nadmm_vec.hip"]:
        with open(os.path.join(here, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:12]


def measured_traffic(name, path):
    ent = MEASURED_HV_TRAFFIC.get((name, path))
    if ent is None:
        return None, None
    nbytes, profile, digest = ent
    cur = source_digest(path)
    if digest != cur:
        return None, f"{profile} was measured with kernel sources {digest or '(unrecorded)'}; they are {cur} now"
    return nbytes, f"{profile} (kernel sources {digest})"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="image_like")
    ap.add_argument("--n", type=int, default=None, help="override the number of rows (testing only)")
    ap.add_argument("--path", type=int, default=0,
                    help="kernel path: 0 auto, 1 two-pass, 2 fused, 3 thin, 4 column-sliced, 5 sparse storage")
    ap.add_argument("--admm-workers", type=int, default=4,
                    help="simulated ADMM workers for the outer-iteration timing in extra (0 or 1: skip)")
    ap.add_argument("--admm-outer", type=int, default=2, help="outer iterations timed for that figure")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the measurements outside the timed steps (two copies of A, ADMM): profiling runs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--only", default="", help="comma list of hv,lg,solve: restrict the step (profiling runs)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run 3 plain device copies of A (known size) so that HBM counters can be scaled")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the Hessian-vector timing of the other dense benchmark configurations in extra")
    ap.add_argument("--hv-per-step", type=int, default=HV_PER_STEP)
    ap.add_argument("--lg-per-step", type=int, default=LG_PER_STEP)
    return ap.parse_args()


def cpu_baseline(w, seconds):
    """The float64 oracle's Hessian-vector product, timed on the host cores as it stands."""
    import numpy as np
    from threadpoolctl import threadpool_info

    from oracle import nadmm_oracle as orc

    prob = orc.Problem(w.A, w.b, w.C, s=w.s, lam=w.lam, rho=w.rho, z=w.z, y=w.y)
    X = w.X0.astype(np.float64)
    V = w.V.astype(np.float64)
    orc.hessvec(prob, X, V)  # warm-up (page faults, BLAS thread start)
    reps, t0 = 0, time.perf_counter()
    while True:
        orc.hessvec(prob, X, V)
        reps += 1
        el = time.perf_counter() - t0
        if el >= seconds or reps >= 5000:
            break
    threads = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    avail = len(os.sched_getaffinity(0))
    return {"value": reps / el, "unit": "Hv/s", "cores": min(threads, avail), "kind": "oracle",
            "sample": f"{reps} float64 numpy{'/scipy.sparse' if w.sparse else ''} Hessian-vector products at the "
                      f"full workload shape ({w.n}x{w.p}, C={w.C}) in {el:.1f} s"}


def other_configs(nadmm, workloads, torch, np, skip):
    """Hessian-vector and local-solve times with their HBM fractions for the other dense benchmark configurations
    (outside the timed steps)."""
    out = {}
    for name in ("wide", "tall_binary", "large_multiclass"):
        if name == skip:
            continue
        try:
            w = workloads.make(name, 0)
            gp = nadmm.Problem.from_workload(w)
            ws = gp.workspace()
            X, V, hv = torch.from_numpy(w.X0).cuda(), torch.from_numpy(w.V).cuda(), gp.vec()
            # the GPU has idled while the host generated the data: warm up for about 50 ms of calls before timing 100
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                nadmm.nadmm_hessvec(gp, X, V, out=hv, ws=ws)
            e1.record()
            torch.cuda.synchronize()
            per_call_ms = max(e0.elapsed_time(e1) / 10, 1e-3)
            for _ in range(min(2000, int(50.0 / per_call_ms))):
                nadmm.nadmm_hessvec(gp, X, V, out=hv, ws=ws)
            reps = 100
            e0.record()
            for _ in range(reps):
                nadmm.nadmm_hessvec(gp, X, V, out=hv, ws=ws)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / reps
            nbytes = 4.0 * w.n * w.p + 12.0 * w.p * (w.C - 1)
            out[w.name] = {"hv_us": us, "hv_hbm_frac": nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                           "kernel_path": nadmm.nadmm_query_kernel_path(gp)}
            # one local Newton-CG solve at the workload's iteration budget (after one untimed solve), against the HBM
            # time of the method's passes over A, as extra.local_solve_hbm_frac does for the headline workload
            params = nadmm.make_params(w.max_newton, w.max_cg, w.max_ls, 0.0, 0.0, w.beta, w.gamma)
            ws = gp.workspace(params)
            X0 = torch.from_numpy(w.X0).cuda()
            Xs = X0.clone()
            nadmm.nadmm_local_newton(gp, Xs, params, want_stats=False, ws=ws)
            Xs.copy_(X0)
            e0.record()
            nadmm.nadmm_local_newton(gp, Xs, params, want_stats=False, ws=ws)
            e1.record()
            torch.cuda.synchronize()
            solve_s = e0.elapsed_time(e1) / 1e3
            passes = w.max_newton * (w.max_cg + 2)
            out[w.name].update({"local_solve_seconds": solve_s, "local_solve_passes_over_A": passes,
                                "local_solve_hbm_frac": passes * 4.0 * w.n * w.p / solve_s / 1e9 / HBM_PEAK_GBS})
            del gp, ws, w
            torch.cuda.empty_cache()
        except Exception as e:  # never lose the headline line over an extra
            out[name] = {"error": repr(e)[:200]}
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (one ADMM worker's data share); "
              "--gpus above 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_1807_07132_amd import nadmm, workloads

    torch.cuda.set_device(0)
    w = workloads.make(args.workload, 0, args.n)
    gp = nadmm.Problem.from_workload(w)
    nadmm.nadmm_set_kernel_path(args.path)
    path = nadmm.nadmm_query_kernel_path(gp)
    rng = np.random.default_rng(1234)
    Vs = [torch.from_numpy(rng.standard_normal(w.V.shape).astype(np.float32)).cuda() for _ in range(4)]
    X = torch.from_numpy(w.X0).cuda()
    hv_out = gp.vec()
    g_out = gp.vec()
    loss_out = torch.empty((), dtype=torch.float64, device="cuda")
    params = nadmm.make_params(w.max_newton, w.max_cg, w.max_ls, 0.0, 0.0, w.beta, w.gamma)
    ws = gp.workspace(params)   # sized for the local solve: every entry point accepts it
    Xs = gp.vec()
    only = set(x for x in args.only.split(",") if x)
    do = lambda k: not only or k in only

    ev = lambda: torch.cuda.Event(enable_timing=True)

    def step():
        t = {}
        if do("hv"):
            e0, e1 = ev(), ev()
            e0.record()
            for i in range(args.hv_per_step):
                nadmm.nadmm_hessvec(gp, X, Vs[i & 3], out=hv_out, ws=ws)
            e1.record()
            t["hv"] = (e0, e1)
        if do("lg"):
            e0, e1 = ev(), ev()
            e0.record()
            for i in range(args.lg_per_step):
                nadmm.nadmm_loss_grad(gp, X, loss_out=loss_out, grad_out=g_out, ws=ws)
            e1.record()
            t["lg"] = (e0, e1)
        if do("solve"):
            Xs.copy_(X)
            e0, e1 = ev(), ev()
            e0.record()
            nadmm.nadmm_local_newton(gp, Xs, params, want_stats=False, ws=ws)
            e1.record()
            t["solve"] = (e0, e1)
        return t

    if args.copy_calibration:
        src = gp.A.tensors[2] if w.sparse else gp.A       # sparse storage: the value array of the row view
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    recs = [step() for _ in range(args.steps)]
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms = {k: [r[k][0].elapsed_time(r[k][1]) for r in recs] for k in recs[0]} if recs else {}

    # Outside the timed steps: matrices that fit the 256 MB Infinity Cache are also timed with two
    # independent copies of A used in turn, so that every call has to read its A from HBM.
    cold_hv_us = None
    if do("hv") and recs and not args.no_extras and not w.sparse and gp.A.numel() * 4 < 256e6:
        gp2 = nadmm.Problem(gp.A.clone(), gp.labels, w.C, w.s, w.lam, w.rho, gp.z, gp.y)
        pair = (gp, gp2)
        for i in range(8):
            nadmm.nadmm_hessvec(pair[i & 1], X, Vs[i & 3], out=hv_out, ws=ws)
        e0, e1 = ev(), ev()
        e0.record()
        for i in range(args.hv_per_step):
            nadmm.nadmm_hessvec(pair[i & 1], X, Vs[i & 3], out=hv_out, ws=ws)
        e1.record()
        torch.cuda.synchronize()
        cold_hv_us = e0.elapsed_time(e1) * 1e3 / args.hv_per_step
        del gp2, pair
    tot = {k: sum(v) for k, v in ms.items()}

    # Outside the timed steps: Algorithm 1 with the rows of A split over simulated workers (one after the
    # other on this GPU, fixed penalty): time of one outer iteration and of the consensus step alone.
    admm = None
    if args.admm_workers > 1 and not only and not args.no_extras:
        N = args.admm_workers
        bounds = [w.n * i // N for i in range(N + 1)]
        if w.sparse:
            rows = [w.A[bounds[i]:bounds[i + 1]] for i in range(N)]
            mats = [nadmm.SparseA.from_scipy(r, r.tocsc()) for r in rows]
        else:
            mats = [gp.A[bounds[i]:bounds[i + 1]] for i in range(N)]
        shards = [nadmm.Problem(mats[i], gp.labels[bounds[i]:bounds[i + 1]], w.C, w.s, 0.0, w.rho) for i in range(N)]
        ap = nadmm.make_admm_params(args.admm_outer, params)
        aws = torch.empty(nadmm.nadmm_admm_workspace_bytes(shards, ap), dtype=torch.uint8, device="cuda")
        xw = torch.stack([X] * N).contiguous()
        nadmm.nadmm_admm_solve(shards, w.lam, xw, ap, want_stats=False, ws=aws)   # warm-up
        xw.copy_(torch.stack([X] * N))
        e0, e1 = ev(), ev()
        e0.record()
        nadmm.nadmm_admm_solve(shards, w.lam, xw, ap, want_stats=False, ws=aws)
        e1.record()
        torch.cuda.synchronize()
        t_admm = e0.elapsed_time(e1) / 1e3 / args.admm_outer
        uw, zw = torch.zeros_like(xw), torch.zeros_like(X)
        for _ in range(3):
            nadmm.nadmm_admm_consensus(xw, uw, zw, [w.rho] * N, w.lam, ws=aws)
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(20):
            nadmm.nadmm_admm_consensus(xw, uw, zw, [w.rho] * N, w.lam, ws=aws)
        e1.record()
        torch.cuda.synchronize()
        admm = {"workers": N, "outer_iterations_timed": args.admm_outer, "seconds_per_outer_iteration": t_admm,
                "consensus_step_us": e0.elapsed_time(e1) * 1e3 / 20}
        if not w.sparse:
            # outer iterations until the residual test stops the solver, from the workload's penalty: kept fixed, and
            # adapted by residual balancing (mu = 10, tau = 2)
            eps_abs, eps_rel, cap = 1e-4, 1e-3, 64
            runs = {}
            for name, rule in (("fixed_penalty", 0), ("residual_balancing", 1)):
                apr = nadmm.make_admm_params(cap, params, eps_abs, eps_rel, penalty_rule=rule)
                xw.copy_(torch.stack([X] * N))
                e0, e1 = ev(), ev()
                e0.record()
                _, _, st = nadmm.nadmm_admm_solve(shards, w.lam, xw, apr, ws=aws)
                e1.record()
                torch.cuda.synchronize()
                runs[name] = {"outer_iterations": st["outer_iters"], "stopped_by_residual_test": st["converged"],
                              "seconds": e0.elapsed_time(e1) / 1e3,
                              "final_penalty_factor": st["rho_scale"]}
            admm["to_tolerance"] = {"eps_abs": eps_abs, "eps_rel": eps_rel, "max_outer": cap, **runs}
        del shards, aws, xw, uw, zw

    n, p, NC = w.n, w.p, w.C - 1
    d = p * NC
    # algorithmic bytes: one read of A (sparse storage: the values and column indices of the row view and its
    # row pointers, once) plus the vectors in and out
    bytes_A = (8.0 * w.A.nnz + 8.0 * (n + 1)) if w.sparse else 4.0 * n * p
    entries = float(w.A.nnz) if w.sparse else float(n) * p
    bytes_hv = bytes_A + 3 * 4.0 * d
    bytes_lg = bytes_A + 4.0 * n + 4 * 4.0 * d
    extra = {"kernel_path": {1: "two-pass fp32 vector kernels", 2: "fused single pass (matrix cores)",
                             3: "thin-data single pass", 4: "column-sliced two sweeps (matrix cores)",
                             5: "sparse storage: row view, then column view"}[path]}
    if w.sparse:
        extra["stored_entries"] = int(w.A.nnz)
    value = None
    roof = None
    if "hv" in tot:
        per_hv_s = tot["hv"] / 1e3 / (args.hv_per_step * args.steps)
        value = 1.0 / per_hv_s
        ach = bytes_hv / per_hv_s / 1e9
        traffic, traffic_source = measured_traffic(w.name, path)
        roof = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                "traffic": traffic, "traffic_source": traffic_source,
                "kernel": "Hessian-vector product (all kernels of one nadmm_hessvec call)",
                "us_per_launch": per_hv_s * 1e6, "algorithmic_bytes": bytes_hv}
        extra["hv_us"] = per_hv_s * 1e6
        flops = 4.0 * entries * NC  # useful flops of one Hessian-vector product (the logits A X are overhead)
        extra["hv_tflops_useful"] = flops / per_hv_s / 1e12
        extra["hv_frac_fp32_vector_peak"] = flops / per_hv_s / 1e12 / 157.3
        if cold_hv_us is not None:
            # A fits the Infinity Cache; with two copies used in turn every call has to read its A from HBM
            roof["us_per_launch_two_copies_of_A"] = cold_hv_us
            roof["frac_two_copies_of_A"] = bytes_hv / (cold_hv_us * 1e-6) / 1e9 / HBM_PEAK_GBS
            extra["hv_us_two_copies_of_A"] = cold_hv_us
            extra["hv_hbm_frac_two_copies_of_A"] = bytes_hv / (cold_hv_us * 1e-6) / 1e9 / HBM_PEAK_GBS
    if "lg" in tot:
        per_lg_s = tot["lg"] / 1e3 / (args.lg_per_step * args.steps)
        extra["loss_grad_per_s"] = 1.0 / per_lg_s
        extra["loss_grad_us"] = per_lg_s * 1e6
        extra["loss_grad_hbm_frac"] = bytes_lg / per_lg_s / 1e9 / HBM_PEAK_GBS
    if "solve" in tot:
        per_solve_s = tot["solve"] / 1e3 / args.steps
        passes = w.max_newton * (w.max_cg + 2)
        extra["local_solve_seconds"] = per_solve_s
        extra["local_solve_passes_over_A"] = passes
        extra["local_solve_hbm_frac"] = passes * bytes_A / per_solve_s / 1e9 / HBM_PEAK_GBS
        # the method's passes (gradient, max_cg Hessian-vector products, A p per Newton iteration) against the ones the
        # library makes: with a workspace sized for the parameters the fused path keeps the A d_k of its CG sweeps and
        # puts A p together from them
        kept = nadmm.nadmm_workspace_bytes(gp, params) > nadmm.nadmm_workspace_bytes(gp)
        made = w.max_newton * (w.max_cg + (1 if kept else 2))
        extra["local_solve_passes_over_A_made"] = made
        extra["local_solve_hbm_frac_of_passes_made"] = made * bytes_A / per_solve_s / 1e9 / HBM_PEAK_GBS

    if admm is not None:
        extra["admm"] = admm
    if not only and not args.no_extras and not args.no_other_configs and not w.sparse and args.n is None:
        del gp, ws
        torch.cuda.empty_cache()
        extra["other_configs"] = other_configs(nadmm, workloads, torch, np, args.workload)
    out = {
        "metric": f"Hv products/s ({w.name}: n={n}, p={p}, C={w.C}); loss+grad/s and local Newton-CG solve seconds in extra",
        "value": value, "unit": "Hv/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / max(args.steps, 1), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": DTYPE, "data": "synthetic",
        "config": {"workload": w.name, "n": n, "p": p, "C": w.C, "hv_per_step": args.hv_per_step,
                   "loss_grad_per_step": args.lg_per_step, "newton_iters": w.max_newton, "cg_iters": w.max_cg,
                   "loss_scale": "1/n", "lambda": w.lam, "rho": w.rho},
        "roofline": roof, "extra": extra,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
