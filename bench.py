#!/usr/bin/env python3
"""Benchmark: ADMM iterations/s of the pdADMM-G hot path (all layers) on one MI355X.

One step = one full iteration of Algorithm 1 over every layer (p, W, b, z, q, u updates with their
backtracking) on a synthetic workload whose inputs are resident in HBM before timing starts.
Prints ONE JSON line with the metric, the roofline of the dominant kernel (the fp32 MFMA product
kernel, timed per launch with HIP events on the library's stream during the timed region) and the
CPU oracle timed on the host cores on one iteration of the same workload.
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

MFMA_FP32_PEAK_TFLOPS = 157.3      # MI355X dense fp32 matrix peak
HBM_PEAK_GBS = 8000.0

# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc runs (FETCH_SIZE / WRITE_SIZE scaled
# by a copy kernel of known size); see profiles/. None until measured for a workload.
MEASURED_TRAFFIC_BYTES = {"C2": 1.74e9, "C3": 4.17e10}   # FETCH_SIZE + WRITE_SIZE per launch, profiles/<workload>_iteration_kernels.md


def gemm_flops_per_iteration(dims, n_nodes):
    """Algorithmic flops of the dense products of one iteration, per kernel class:
    layer 1 has no p-update (2 products), every layer l >= 2 has 4; each is 2*n_l*n_{l-1}*|V|."""
    L = len(dims) - 1
    per = [2.0 * dims[i + 1] * dims[i] * n_nodes for i in range(L)]
    return dict(gemm_pgrad=sum(per[1:]),            # W^T r          (l >= 2)
                gemm_trial=sum(per[1:]) + sum(per),  # W g (l >= 2) and G p (all l): two launches
                gemm_wgrad=sum(per))                 # r p^T          (all l)


def elementwise_bytes_per_iteration(dims, n_nodes, quant, fused):
    """Algorithmic HBM bytes of the streaming kernels of one iteration (fp32 arrays of N x n, each counted
    once per read and once per write): fused z/q/u 5 reads + 4 writes over [N, n_l] (l < L); where the
    library applies them in separate kernels also the p-step, 3 passes over [N, n_{l-1}] and 3 over
    [N, n_l] (l >= 2; bit 0 of `fused` clear), and the residual update + column sums, 3 passes over
    [N, n_l] (all l; bit 1 clear). Where a bit is set that update rides in the product epilogues and the
    kernels of its class are corrections that do nothing once the step sizes have settled: no bytes are
    credited to them. The -Q projection kernels are left out (they run a data-dependent number of times)."""
    L = len(dims) - 1
    e = 4.0 * n_nodes
    out = dict(zqu=sum(9 * e * dims[i + 1] for i in range(L - 1)))
    if not fused & 2:
        out["resid_colsum"] = sum(3 * e * dims[i + 1] for i in range(L))
    if not fused & 1 and not quant:
        out["p_step"] = sum(3 * e * (dims[i] + dims[i + 1]) for i in range(1, L))
    return out


def build_problem(w, device, use_graph=0):
    """Inputs -> HBM -> context with a perturbed (generic) state. Uses only the HIP library."""
    import numpy as np
    import torch
    import paper_2105_09837_amd as P
    from workloads import (make_features, make_graph, make_labels, make_weights, perturb_state, stream_rng)

    t0 = time.perf_counter()
    rp, ci = make_graph(w.graph, w.n_nodes, w.graph_param, stream_rng(w, 0))
    a_rp, a_ci, a_v = P.pdadmm_normalize_adj(rp, ci)
    X = make_features(w)
    Ws, bs = make_weights(w)
    y = make_labels(w)
    t1 = time.perf_counter()
    Xd = torch.from_numpy(X).to(device)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    csr = [torch.from_numpy(a).to(device) for a in (a_rp, a_ci, a_v)]
    e0.record()
    Xa = P.pdadmm_augment(csr[0], csr[1], csr[2], Xd, w.hops)
    e1.record()
    torch.cuda.synchronize()
    aug_ms = e0.elapsed_time(e1)
    q = w.quant
    cfg = P.Config(n_nodes=w.n_nodes, dims=list(w.dims), rho=w.rho, nu=w.nu, quantize=(2 if w.quant_q else 1) if q else 0,
                   q_lo=q[0] if q else -1.0, q_hi=q[1] if q else 1.0, q_levels=q[2] if q else 256,
                   use_graph=use_graph)
    ctx = P.pdadmm_init(cfg, Xa, torch.from_numpy(y).to(device), [torch.from_numpy(a).to(device) for a in Ws],
                        [torch.from_numpy(a).to(device) for a in bs])
    # perturb the forward-consistent start (otherwise most layers sit at a fixed point for many iterations)
    L = w.n_layers
    z = [P.pdadmm_get_var(ctx, P.VAR.Z, l + 1) for l in range(L)]
    qs = [P.pdadmm_get_var(ctx, P.VAR.Q, l + 1) for l in range(L - 1)]
    z2, q2, p2, u2 = perturb_state(w, z, qs)
    for l in range(L):
        P.pdadmm_set_var(ctx, P.VAR.Z, l + 1, z2[l])
        if l < L - 1:
            P.pdadmm_set_var(ctx, P.VAR.Q, l + 1, q2[l])
            P.pdadmm_set_var(ctx, P.VAR.P, l + 2, p2[l])       # projected onto the grid by the library in -Q
            P.pdadmm_set_var(ctx, P.VAR.U, l + 1, u2[l])
    info = dict(host_gen_s=t1 - t0, augment_ms=aug_ms, nnz=int(a_ci.size))
    host = dict(rowptr=rp, colidx=ci, X=X, W=Ws, b=bs, y=y)
    return ctx, info, host


def cpu_baseline(w, host):
    """The oracle, as it stands, on one iteration of the same workload (bounded sample)."""
    import numpy as np
    from oracle import pdadmm_oracle as O
    from workloads import perturb_state
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    arp, aci, av = O.normalize_adj(host["rowptr"], host["colidx"])
    Xa = O.augment(arp, aci, av, host["X"], w.hops)
    grid = O.Grid(*w.quant) if w.quant else None
    st = O.init_forward(Xa, host["W"], host["b"], host["y"], w.rho, w.nu, grid=grid, quantize_q=w.quant_q)
    quant = (lambda a: O.quantize(a, grid)[1]) if grid else None
    z, q, p, u = perturb_state(w, [a.astype(np.float32) for a in st.z], [a.astype(np.float32) for a in st.q],
                               quantizer=quant)
    for i in range(st.L):
        st.z[i] = z[i].astype(np.float64)
        if i < st.L - 1:
            st.q[i], st.p[i + 1], st.u[i] = (a[i].astype(np.float64) for a in (q, p, u))
            if w.quant_q:
                st.q[i] = quant(q[i]).astype(np.float64)
    t0 = time.perf_counter()
    O.iterate(st, 1)
    dt = time.perf_counter() - t0
    model = ""
    try:
        with open("/proc/cpuinfo") as f:
            model = next((ln.split(":", 1)[1].strip() for ln in f if ln.startswith("model name")), "")
    except OSError:
        pass
    return dict(value=1.0 / dt, unit="iterations/s", cores=int(threads), kind="oracle",
                sample=f"1 iteration of {w.name} (all {st.L} layers, fp64 numpy), {dt:.1f} s",
                cpu_model=model, os_cpu_count=os.cpu_count())


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10,
                    help="untimed iterations first (default 10: by then the step sizes tau, theta of the perturbed start have settled)")
    ap.add_argument("--workload", default="C2", help="C1..C5, C5pq (default C2: the configuration the metric is quoted on)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--dominant-only", action="store_true",
                    help="record HIP events around the dominant kernel class only (default: every class)")
    ap.add_argument("--graph", action="store_true",
                    help="replay the iteration as a HIP graph (pdADMM-G only; per-class timing is then off)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (reference point for FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2105_09837_amd as P
    from workloads import get_workload

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    P.load_library()
    device = torch.device("cuda:0")
    w = get_workload(args.workload)
    ctx, info, host = build_problem(w, device, use_graph=1 if args.graph else 0)

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=device)      # 1 GiB
        dst = torch.empty_like(src)
        torch.add(src, 1.0, out=dst)                                       # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    P.pdadmm_iterate(ctx, args.warmup)
    P.pdadmm_sync(ctx)
    dominant = "gemm_trial"
    mask = 1 << P.TIMING_CLASSES.index(dominant) if args.dominant_only else (1 << len(P.TIMING_CLASSES)) - 1
    if args.graph:
        mask = 0                       # events around single launches would break the replay up
    P.pdadmm_timing(ctx, mask)
    products_before = P.pdadmm_stats(ctx)["p_products"]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    P.pdadmm_iterate(ctx, args.steps)
    P.pdadmm_sync(ctx)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    timing = P.pdadmm_timing_read(ctx)
    P.pdadmm_timing(ctx, 0)
    stats = P.pdadmm_stats(ctx)
    plan = P.pdadmm_plan_info(ctx)
    obj = P.pdadmm_objective(ctx)

    flops = gemm_flops_per_iteration(w.dims, w.n_nodes)
    ms, launches = timing[dominant]
    launches_per_iter = launches / max(args.steps, 1)
    # step-direction products actually computed (pdADMM-G: one per layer l >= 2 and iteration; -Q: one per
    # backtracking trial of the layer; layers whose search has ended sit out the later launches) plus the
    # G p products of all layers
    n_products = stats["p_products"] - products_before
    per_layer = [2.0 * w.dims[i + 1] * w.dims[i] * w.n_nodes for i in range(w.n_layers)]
    trial_flops = (sum(float(n_products[i]) * per_layer[i] for i in range(w.n_layers)) / max(args.steps, 1)
                   + sum(per_layer))
    flops_per_launch = trial_flops / launches_per_iter if launches_per_iter else 0.0
    avg_ms = ms / launches if launches else None
    achieved = flops_per_launch / (avg_ms * 1e-3) / 1e12 if launches else None
    roofline = dict(bound="mfma", kernel="gemm_kernel<NT, EpiTrialP|EpiTrialW|EpiStoreNorm> (fp32 MFMA 32x32x2; W g / W d and G p products)",
                    achieved=achieved, peak=MFMA_FP32_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=achieved / MFMA_FP32_PEAK_TFLOPS if achieved else None,
                    traffic=MEASURED_TRAFFIC_BYTES.get(w.name), avg_launch_ms=avg_ms, launches=launches,
                    flop_per_launch=flops_per_launch)
    total_gemm_flops = flops["gemm_pgrad"] + flops["gemm_wgrad"] + trial_flops
    out = dict(metric="ADMM iterations/sec (all layers)", value=args.steps / dt, unit="iterations/s", n_gpus=1,
               steps=args.steps, warmup=args.warmup, ms_per_step=dt / args.steps * 1e3, higher_is_better=True,
               scaling="weak", vs_baseline=None, dtype="f32", data="synthetic",
               config=dict(workload=f"{w.name}: N={w.n_nodes} {w.graph} graph, X {w.feat_dim}-dim, hops={w.hops} -> n0={w.n0}, "
                                    f"L={w.n_layers}, hidden={w.hidden}, classes={w.n_classes}, rho=nu={w.rho}"
                                    + (f", Delta={w.quant[2]} levels on [{w.quant[0]},{w.quant[1]}]" if w.quant else ""),
                           variant=("pdADMM-G-Q (p and q on the grid)" if w.quant_q else "pdADMM-G-Q") if w.quant else "pdADMM-G"),
               gemm_tflops_whole_iteration=total_gemm_flops * args.steps / dt / 1e12,
               roofline=roofline,
               augment_ms=info["augment_ms"], objective_after=obj["L_rho"],
               p_trials=[int(x) for x in stats["p_trials"]], w_trials=[int(x) for x in stats["w_trials"]],
               plan=dict(fused_updates=plan["fused_updates"], wgrad_split=[int(x) for x in plan["wgrad_split"]],
                         wtrial_split=plan["wtrial_split"]))
    if not args.dominant_only and not args.graph:
        cls = {k: v[0] / args.steps for k, v in timing.items() if v[1]}
        out["class_ms_per_step"] = cls
        gemm_ms = sum(cls.get(k, 0.0) for k in ("gemm_pgrad", "gemm_trial", "gemm_wgrad", "splitk_reduce"))
        launched = total_gemm_flops
        eb = elementwise_bytes_per_iteration(w.dims, w.n_nodes, w.quant, plan["fused_updates"])
        ew_ms = sum(cls.get(k, 0.0) for k in eb)
        out["phases"] = dict(
            gemm=dict(ms=gemm_ms, tflops=launched / (gemm_ms * 1e-3) / 1e12 if gemm_ms else None,
                      frac_of_mfma_peak=launched / (gemm_ms * 1e-3) / 1e12 / MFMA_FP32_PEAK_TFLOPS if gemm_ms else None),
            elementwise=dict(ms=ew_ms, gbs=sum(eb.values()) / (ew_ms * 1e-3) / 1e9 if ew_ms else None,
                             frac_of_hbm_peak=sum(eb.values()) / (ew_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if ew_ms else None,
                             per_kernel_gbs={k: eb[k] / (cls[k] * 1e-3) / 1e9 for k in eb if cls.get(k)}))
        if plan["fused_updates"]:     # what is left of these classes: the step-size corrections
            out["phases"]["corrections_ms"] = ((cls.get("p_step", 0.0) if plan["fused_updates"] & 1 else 0.0)
                                               + (cls.get("resid_colsum", 0.0) if plan["fused_updates"] & 2 else 0.0))
    if not args.no_cpu_baseline:
        del ctx
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(w, host)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
