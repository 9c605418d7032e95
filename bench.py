#!/usr/bin/env python3
"""Benchmark: ADMM iterations/s of the pdADMM-G / pdADMM-G-Q hot path (all layers) on one MI355X.

One step = one full iteration of Algorithm 1 over every layer (p, W, b, z, q, u updates with their
backtracking) on a synthetic workload whose inputs are resident in HBM before timing starts.
Prints ONE JSON line: the metric on the headline workload (default C3, the largest pdADMM-G configuration
that fits one GPU), the roofline of its dominant kernel (the fp32 MFMA product kernel, timed per launch with
HIP events on the library's stream during the timed region), the CPU oracle timed on the host cores on a
bounded sample of the same workload, and under `per_config` the same figures in short for the other
workloads (C5 is the largest pdADMM-G-Q configuration).
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
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")


def measured_traffic(workload):
    """HBM bytes per launch of the dominant kernel class from the rocprofv3 --pmc runs summarised under
    profiles/ (FETCH_SIZE and WRITE_SIZE, each scaled by what the same counter reads for a plain copy kernel
    of known size); None for a workload that has not been profiled."""
    try:
        with open(TRAFFIC_FILE) as f:
            entry = json.load(f).get(workload)
    except (OSError, ValueError):
        return None
    return None if entry is None else float(entry["fetch_bytes_per_launch"]) + float(entry["write_bytes_per_launch"])


def gemm_flops_per_iteration(dims, n_nodes):
    """Algorithmic flops of the dense products of one iteration, per kernel class:
    layer 1 has no p-update (2 products), every layer l >= 2 has 4; each is 2*n_l*n_{l-1}*|V|."""
    L = len(dims) - 1
    per = [2.0 * dims[i + 1] * dims[i] * n_nodes for i in range(L)]
    return dict(gemm_pgrad=sum(per[1:]),            # W^T r          (l >= 2)
                gemm_trial=sum(per[1:]) + sum(per),  # W g (l >= 2) and G p (all l): two launches
                gemm_wgrad=sum(per))                 # r p^T          (all l)


def elementwise_bytes_per_iteration(dims, n_nodes, quant, fused, trials_per_iter, p_bytes=4):
    """Algorithmic HBM bytes of the streaming kernels of one iteration, per timing class (fp32 arrays of
    N x n, each counted once per read and once per write):
      zqu           fused z/q/u: reads r, z, q, u (4 B each) and p_{l+1} (p_bytes), writes z, r, q, u over
                    [N, n_l], l < L;
      p_step        pdADMM-G, where not folded into the product epilogues (bit 0 of `fused` clear): 3 passes
                    over [N, n_{l-1}] and 3 over [N, n_l], l >= 2;
      resid_colsum  r -= Gp/theta with column sums, 3 passes over [N, n_l], all l (bit 1 clear);
      quant_trial   -Q: per backtracking trial of a layer, reads p_l (p_bytes) and g, writes d (4 B) and the
                    candidate index (1 B, 2 B above 256 levels) over [N, n_{l-1}]; `trials_per_iter[l-1]` = measured trials per
                    iteration of layer l;
      quant_apply   -Q, per layer and iteration: what the library does on acceptance (p_l <- Delta[idx]:
                    1 B read + 4 B written per element while p_l is kept as fp32, nothing once p_l is kept as
                    indices) plus r += W d, 3 passes over [N, n_l].
    Where a bit of `fused` is set that update rides in the product epilogues and the kernels of its class
    are corrections that do nothing once the step sizes have settled: no bytes are credited to them."""
    L = len(dims) - 1
    e = float(n_nodes)
    out = dict(zqu=sum((8 * 4 + p_bytes) * e * dims[i + 1] for i in range(L - 1)))
    if not fused & 2:
        out["resid_colsum"] = sum(12 * e * dims[i + 1] for i in range(L))
    if not fused & 1 and not quant:
        out["p_step"] = sum(12 * e * (dims[i] + dims[i + 1]) for i in range(1, L))
    if quant:
        idx_bytes = p_bytes if p_bytes < 4 else 1        # width of a stored index (2 above 256 levels)
        out["quant_trial"] = sum(trials_per_iter[i] * (p_bytes + 4 + 4 + idx_bytes) * e * dims[i] for i in range(1, L))
        apply_p = (1 + 4) if p_bytes == 4 else 0
        out["quant_apply"] = sum(apply_p * e * dims[i] + 12 * e * dims[i + 1] for i in range(1, L))
    return out


def build_problem(w, device, use_graph=0, backoff=1, streams=None):
    """Inputs -> HBM -> context with a perturbed (generic) state. Uses only the HIP library."""
    import torch
    import paper_2105_09837_amd as P
    from workloads import (make_features, make_graph, make_labels, make_weights, perturb_layers, stream_rng)

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
    Xa = P.pdadmm_augment(csr[0], csr[1], csr[2], Xd, w.hops)      # first launch of the library: loads its code object
    torch.cuda.synchronize()
    e0.record()
    Xa = P.pdadmm_augment(csr[0], csr[1], csr[2], Xd, w.hops, out=Xa)
    e1.record()
    torch.cuda.synchronize()
    aug_ms = e0.elapsed_time(e1)
    q = w.quant
    cfg = P.Config(n_nodes=w.n_nodes, dims=list(w.dims), rho=w.rho, nu=w.nu, quantize=(2 if w.quant_q else 1) if q else 0,
                   q_lo=q[0] if q else -1.0, q_hi=q[1] if q else 1.0, q_levels=q[2] if q else 256,
                   use_graph=use_graph, bt_probe_backoff=backoff, risk_kind=P.RISK[w.risk])
    yd, Wd, bd = torch.from_numpy(y).to(device), [torch.from_numpy(a).to(device) for a in Ws], [torch.from_numpy(a).to(device) for a in bs]
    torch.cuda.synchronize()
    ctx = P.pdadmm_init(cfg, Xa, yd, Wd, bd, stream=streams[0] if streams else None,
                        aux_stream=streams[1] if streams and len(streams) > 1 else None)
    # perturb the forward-consistent start (otherwise most layers sit at a fixed point for many iterations)
    L = w.n_layers

    class Lazy:     # z_l, q_l are fetched from the device when the perturbation reaches layer l
        def __init__(self, kind, n):
            self.kind, self.n = kind, n

        def __len__(self):
            return self.n

        def __getitem__(self, l):
            return P.pdadmm_get_var(ctx, self.kind, l + 1)

    for l, z2, q2, p2, u2 in perturb_layers(w, Lazy(P.VAR.Z, L), Lazy(P.VAR.Q, L - 1)):
        P.pdadmm_set_var(ctx, P.VAR.Z, l + 1, z2)
        if l < L - 1:
            P.pdadmm_set_var(ctx, P.VAR.Q, l + 1, q2)
            P.pdadmm_set_var(ctx, P.VAR.P, l + 2, p2)       # projected onto the grid by the library in -Q
            P.pdadmm_set_var(ctx, P.VAR.U, l + 1, u2)
    info = dict(host_gen_s=t1 - t0, augment_ms=aug_ms, nnz=int(a_ci.size), build_s=time.perf_counter() - t0)
    host = dict(rowptr=rp, colidx=ci, X=X, W=Ws, b=bs, y=y)
    return ctx, info, host


# seconds of oracle time per (node x weight) of one iteration, measured on C2 (11.8 s for 20 000 nodes x 3.0e6
# weights on 16 threads): only used to size the sample below
ORACLE_S_PER_NODE_WEIGHT = 2.0e-10
CPU_BASELINE_BUDGET_S = 15.0


def cpu_baseline(w, host):
    """The oracle, as it stands, timed on ONE iteration over ALL layers of the same workload restricted to
    its first n_s nodes (rows of X_aug and labels; every update of the method works node by node except the
    sums over nodes behind W, b and the step sizes, so the cost is proportional to the number of nodes up to
    the weight-sized terms, which favour the full size). n_s is chosen so that the iteration takes about
    CPU_BASELINE_BUDGET_S; the rate is scaled by n_s / N to the full workload. Workloads small enough run whole."""
    import numpy as np
    from oracle import pdadmm_oracle as O
    from workloads import perturb_state
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    weights = sum(w.dims[i] * w.dims[i + 1] for i in range(w.n_layers))
    n_s = int(CPU_BASELINE_BUDGET_S / (ORACLE_S_PER_NODE_WEIGHT * weights))
    n_s = w.n_nodes if n_s >= w.n_nodes else max(1000, n_s // 1000 * 1000)
    arp, aci, av = O.normalize_adj(host["rowptr"], host["colidx"])
    Xa = O.augment(arp, aci, av, host["X"], w.hops)[:n_s]
    y = host["y"][:n_s]
    grid = O.Grid(*w.quant) if w.quant else None
    st = O.init_forward(Xa, host["W"], host["b"], y, w.rho, w.nu, grid=grid, quantize_q=w.quant_q, risk_kind=w.risk)
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
    scale = n_s / w.n_nodes
    whole = n_s == w.n_nodes
    return dict(value=scale / dt, unit="iterations/s", cores=int(threads), kind="oracle",
                sample=(f"1 iteration of {w.name} (all {st.L} layers, fp64 numpy), {dt:.1f} s" if whole else
                        f"1 iteration over all {st.L} layers of {w.name} restricted to its first {n_s} of {w.n_nodes} nodes "
                        f"(fp64 numpy, the first iteration from the perturbed start), {dt:.1f} s; rate scaled by {n_s}/{w.n_nodes}"),
                cpu_model=model, os_cpu_count=os.cpu_count())


def measure(name, args, device, want_host=False):
    """Build workload `name`, run warm-up + timed iterations, return (result dict, workload, host arrays)."""
    import torch
    import paper_2105_09837_amd as P
    from workloads import get_workload

    w = get_workload(name)
    backoff = 0 if args.plain_schedule else 1
    streams = [torch.cuda.Stream() for _ in range(args.streams)] if args.streams > 1 else None
    ctx, info, host = build_problem(w, device, use_graph=1 if args.graph else 0, backoff=backoff, streams=streams)
    if not want_host:
        host = None
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
    trials_per_iter = [float(n_products[i]) / max(args.steps, 1) for i in range(w.n_layers)]
    per_layer = [2.0 * w.dims[i + 1] * w.dims[i] * w.n_nodes for i in range(w.n_layers)]
    trial_flops = sum(trials_per_iter[i] * per_layer[i] for i in range(w.n_layers)) + sum(per_layer)
    flops_per_launch = trial_flops / launches_per_iter if launches_per_iter else 0.0
    avg_ms = ms / launches if launches else None
    achieved = flops_per_launch / (avg_ms * 1e-3) / 1e12 if launches else None
    roofline = dict(bound="mfma", kernel="gemm_kernel<NT, EpiTrialP|EpiTrialW|EpiStoreNorm> (fp32 MFMA 32x32x2; W g / W d and G p products)",
                    achieved=achieved, peak=MFMA_FP32_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=achieved / MFMA_FP32_PEAK_TFLOPS if achieved else None,
                    traffic=measured_traffic(w.name), avg_launch_ms=avg_ms, launches=launches,
                    flop_per_launch=flops_per_launch)
    total_gemm_flops = flops["gemm_pgrad"] + flops["gemm_wgrad"] + trial_flops
    variant = "pdADMM-G"
    if w.quant:
        variant = ("pdADMM-G-Q (p and q on the grid)" if w.quant_q else "pdADMM-G-Q") + \
                  (", tau/eta probed with back-off" if backoff else ", plain schedule (every update starts at tau/eta)")
    out = dict(metric="ADMM iterations/sec (all layers)", value=args.steps / dt, unit="iterations/s", n_gpus=1,
               steps=args.steps, warmup=args.warmup, ms_per_step=dt / args.steps * 1e3, higher_is_better=True,
               scaling="weak", vs_baseline=None, dtype="f32", data="synthetic",
               config=dict(workload=f"{w.name}: N={w.n_nodes} {w.graph} graph, X {w.feat_dim}-dim, hops={w.hops} -> n0={w.n0}, "
                                    f"L={w.n_layers}, hidden={w.hidden}, classes={w.n_classes}, rho=nu={w.rho}"
                                    + (f", Delta={w.quant[2]} levels on [{w.quant[0]},{w.quant[1]}]" if w.quant else ""),
                           variant=variant, streams=args.streams),
               gemm_tflops_whole_iteration=total_gemm_flops * args.steps / dt / 1e12,
               roofline=roofline,
               augment_ms=info["augment_ms"], build_s=info["build_s"], objective_after=obj["L_rho"],
               p_trials=[int(x) for x in stats["p_trials"]], w_trials=[int(x) for x in stats["w_trials"]],
               plan=dict(fused_updates=plan["fused_updates"], wgrad_split=[int(x) for x in plan["wgrad_split"]],
                         wtrial_split=plan["wtrial_split"]))
    if w.quant:
        out["p_trial_products_per_update"] = sum(trials_per_iter[1:]) / max(w.n_layers - 1, 1)
    if not args.dominant_only and not args.graph:
        cls = {k: v[0] / args.steps for k, v in timing.items() if v[1]}
        out["class_ms_per_step"] = cls
        gemm_ms = sum(cls.get(k, 0.0) for k in ("gemm_pgrad", "gemm_trial", "gemm_wgrad", "splitk_reduce"))
        launched = total_gemm_flops
        eb = elementwise_bytes_per_iteration(w.dims, w.n_nodes, w.quant, plan["fused_updates"], trials_per_iter,
                                             p_bytes=plan.get("p_bytes", 4))
        ew_ms = sum(cls.get(k, 0.0) for k in eb)
        out["phases"] = dict(
            gemm=dict(ms=gemm_ms, tflops=launched / (gemm_ms * 1e-3) / 1e12 if gemm_ms else None,
                      frac_of_mfma_peak=launched / (gemm_ms * 1e-3) / 1e12 / MFMA_FP32_PEAK_TFLOPS if gemm_ms else None),
            elementwise=dict(ms=ew_ms, gbs=sum(eb.values()) / (ew_ms * 1e-3) / 1e9 if ew_ms else None,
                             frac_of_hbm_peak=sum(eb.values()) / (ew_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if ew_ms else None,
                             kernels=sorted(eb),
                             per_kernel_gbs={k: eb[k] / (cls[k] * 1e-3) / 1e9 for k in eb if cls.get(k)}))
        if plan["fused_updates"]:     # what is left of these classes: the step-size corrections
            out["phases"]["corrections_ms"] = ((cls.get("p_step", 0.0) if plan["fused_updates"] & 1 else 0.0)
                                               + (cls.get("resid_colsum", 0.0) if plan["fused_updates"] & 2 else 0.0))
    P.pdadmm_destroy(ctx)
    del ctx
    torch.cuda.empty_cache()
    return out, w, host


def short(res):
    """The per_config entry of a workload: rate and the two phase fractions."""
    ph = res.get("phases", {})
    return dict(workload=res["config"]["workload"].split(":")[0], variant=res["config"]["variant"],
                iterations_per_s=res["value"], ms_per_step=res["ms_per_step"],
                dominant_kernel_frac_of_mfma_peak=res["roofline"]["frac"],
                gemm_phase_frac_of_mfma_peak=ph.get("gemm", {}).get("frac_of_mfma_peak"),
                elementwise_phase_frac_of_hbm_peak=ph.get("elementwise", {}).get("frac_of_hbm_peak"),
                elementwise_kernels=ph.get("elementwise", {}).get("kernels"),
                p_trial_products_per_update=res.get("p_trial_products_per_update"))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10,
                    help="untimed iterations first (default 10: by then the step sizes tau, theta of the perturbed start have settled)")
    ap.add_argument("--workload", default="C3",
                    help="C1..C5, C5pq (default C3: the largest pdADMM-G configuration that fits one GPU)")
    ap.add_argument("--per-config", default="C5,C2,C4,C1",
                    help="other workloads measured after the headline one and reported in short under per_config "
                         "(comma separated, '' for none; a workload is skipped once the run has used --per-config-budget seconds)")
    ap.add_argument("--per-config-budget", type=float, default=200.0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--plain-schedule", action="store_true",
                    help="-Q: every p-update starts at tau/eta (bt_probe_backoff = 0) instead of the probe back-off")
    ap.add_argument("--streams", type=int, default=1, choices=(1, 2),
                    help="2: give the library a second stream for the independent parts of an iteration")
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

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    P.load_library()
    device = torch.device("cuda:0")
    t_start = time.perf_counter()
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=device)      # 1 GiB
        dst = torch.empty_like(src)
        torch.add(src, 1.0, out=dst)                                       # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    out, w, host = measure(args.workload, args, device, want_host=not args.no_cpu_baseline)
    print(f"bench.py: {args.workload} {out['value']:.3f} it/s after {time.perf_counter() - t_start:.0f} s", file=sys.stderr, flush=True)
    per = []
    for name in [n for n in args.per_config.split(",") if n and n != args.workload]:
        if time.perf_counter() - t_start > args.per_config_budget:
            per.append(dict(workload=name, skipped="time budget of this run used up"))
            continue
        res, _, _ = measure(name, args, device)
        per.append(short(res))
        print(f"bench.py: {name} {res['value']:.3f} it/s after {time.perf_counter() - t_start:.0f} s", file=sys.stderr, flush=True)
    if per:
        out["per_config"] = per
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, host)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
