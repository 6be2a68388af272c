#!/usr/bin/env python3
"""Benchmark of the LAGS-SGD hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic gradients that are
already resident in HBM: the per-layer error-compensated top-k sparsifier for all P
workers of the workload (one batched lags_sparsify_model call over P x L layers) and
the merge of the P sparse sets into the dense averaged update (lags_merge_sparse).

Prints ONE JSON line: sparsified elements/s (whole job), the roofline of the dominant
kernel from HIP-event timings taken inside the timed region, and the CPU oracle timed
on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak


def measured_traffic(kernel, workload, workers):
    """HBM bytes per launch of `kernel` for this workload from the committed rocprofv3 counter
    summary (profiles/*.txt, line 'TRAFFIC_BYTES_PER_LAUNCH <kernel> <workload> P=<workers>: <bytes>'),
    or None if no summary covers it."""
    import glob
    key = "TRAFFIC_BYTES_PER_LAUNCH %s %s P=%d:" % (kernel, workload, workers)
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        for line in open(path):
            if line.startswith(key):
                return float(line.split(":")[1])
    return None


def cpu_baseline(wl, grad0_host, threads):
    """The oracle as it stands on the host cores: worker 0, one iteration, every layer,
    layers spread over `threads` host threads."""
    import concurrent.futures as cf
    import numpy as np
    import oracle
    layers = wl.layers()
    res = np.zeros(wl.total_d, np.float32)
    ks = [oracle.topk_count(d, rho) for (_, d, rho) in layers]

    def one(l):
        off, d, _ = layers[l]
        oracle.sparsify_layer(np.ascontiguousarray(grad0_host[off:off + d]), res[off:off + d], wl.lr, ks[l])

    order = sorted(range(len(layers)), key=lambda l: -layers[l][1])
    t0 = time.perf_counter()
    with cf.ThreadPoolExecutor(threads) as ex:
        list(ex.map(one, order))
    dt = time.perf_counter() - t0
    return wl.total_d / dt, dt


def cpu_baseline_extras(wl, grad0_host, idx_host, val_host, P, K):
    """Two more oracle timings for context: the sparsifier on one host thread (the second largest
    layer of worker 0 only, to bound the time) and the merge of the P workers' pairs (one thread)."""
    import numpy as np
    import oracle
    layers = wl.layers()
    order = sorted(range(len(layers)), key=lambda l: -layers[l][1])
    l = order[1] if len(order) > 1 else order[0]
    off, d, rho = layers[l]
    g = np.ascontiguousarray(grad0_host[off:off + d])
    r = np.zeros(d, np.float32)
    t0 = time.perf_counter()
    oracle.sparsify_layer(g, r, wl.lr, oracle.topk_count(d, rho))
    t_one = time.perf_counter() - t0
    upd = np.empty(wl.total_d, np.float32)
    t0 = time.perf_counter()
    oracle.merge_sparse(layers, idx_host, val_host, P, K, upd)
    t_merge = time.perf_counter() - t0
    return {"single_thread_value": d / t_one, "single_thread_sample": "layer %d of worker 0 (%d elements), %.1f s" % (l, d, t_one),
            "merge_value": wl.total_d / t_merge, "merge_unit": "update elements/s",
            "merge_sample": "all %d layers, P = %d, one thread, %.2f s" % (len(layers), P, t_merge)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="vgg16", help="single|resnet20|vgg16|resnet50|lstm")
    ap.add_argument("--rho", default="0.001", help="density for every layer, or 'config' for the workload's own")
    ap.add_argument("--workers", type=int, default=0, help="simulated workers P (0 = the workload's)")
    ap.add_argument("--per-worker", action="store_true",
                    help="one lags_sparsify_model call per worker (L layers each) instead of one batched call")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of 1 GiB (for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path has no inter-GPU step); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_1911_08727_amd import lags, workloads

    dev = torch.device("cuda:0")
    if args.calibrate_copy:
        n = 1 << 28
        a = torch.ones(n, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        for _ in range(args.steps):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "plain copy", "bytes_read": n * 4, "bytes_written": n * 4,
                          "launches": args.steps}))
        return

    rho = None if args.rho == "config" else float(args.rho)
    wl = workloads.make(args.workload, rho_override=rho)
    P = args.workers or wl.P
    total = wl.total_d
    layers = wl.layers()
    batched = [(p * total + off, d, r) for p in range(P) for (off, d, r) in layers]

    ctx = lags.Context(0)
    table_b = ctx.table(batched)      # P x L layers: one sparsify call per step
    table_1 = ctx.table(layers)       # one worker's layout: the merge
    K = table_1.total_k
    assert table_b.total_k == P * K

    grad = torch.empty(P * total, dtype=torch.float32, device=dev)
    for p in range(P):
        workloads.grad_torch(wl, 0, p, dev, out=grad[p * total:(p + 1) * total])
    res = torch.zeros(P * total, dtype=torch.float32, device=dev)
    idx = torch.empty(P * K, dtype=torch.int32, device=dev)
    val = torch.empty(P * K, dtype=torch.float32, device=dev)
    upd = torch.empty(total, dtype=torch.float32, device=dev)
    grad0_host = None if args.no_cpu_baseline else grad[:total].cpu().numpy()
    stream = torch.cuda.current_stream()

    def step():
        if args.per_worker:
            for p in range(P):
                ctx.lags_sparsify_model(table_1, grad[p * total:(p + 1) * total], res[p * total:(p + 1) * total],
                                        wl.lr, idx[p * K:(p + 1) * K], val[p * K:(p + 1) * K], stream)
        else:
            ctx.lags_sparsify_model(table_b, grad, res, wl.lr, idx, val, stream)
        ctx.lags_merge_sparse(table_1, idx, val, P, K, upd, stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # an untimed pass with every kernel bracketed by events: the per-kernel table, and which
    # kernel dominates
    ctx.lags_profile_reset()
    ctx.lags_profile_enable(True)
    n_table = max(2, min(5, args.steps))
    for _ in range(n_table):
        step()
    torch.cuda.synchronize()
    ctx.lags_profile_enable(False)
    prof_all = ctx.lags_profile_read()
    ctx.lags_profile_reset()
    # "sparsify_call" is not a kernel: it brackets the whole sparsify call (fork to join) on the
    # caller's stream; the small layers' kernels on the side stream overlap the streaming pass,
    # so per-kernel times do not add up to it
    call_ms = prof_all.pop("sparsify_call", (0.0, 0))[0] / n_table
    dom = max(prof_all, key=lambda k: prof_all[k][0])
    # the timed region: exactly K steps; only the dominant kernel is bracketed by HIP events
    # (on the stream it is launched on), so the measurement adds two events per step
    ctx.lags_profile_enable_kernel(dom)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ctx.lags_profile_enable(False)
    prof = ctx.lags_profile_read()
    ctx.lags_profile_reset()

    # the rows next to the hot path, measured apart from the timed steps: the in-place sparse
    # parameter step (Algorithm 1 line 9) and the delta metric of Section 6.2
    param = torch.zeros(total, dtype=torch.float32, device=dev)
    delta = torch.empty(3 * len(layers), dtype=torch.float64, device=dev)
    reps = 5
    ctx.lags_apply_sparse(table_1, idx, val, P, K, param, stream)
    ctx.lags_delta_monitor(table_1, res, total, idx, val, P, K, delta, stream)
    torch.cuda.synchronize()
    ctx.lags_profile_enable(True)
    for _ in range(reps):
        ctx.lags_apply_sparse(table_1, idx, val, P, K, param, stream)
        ctx.lags_delta_monitor(table_1, res, total, idx, val, P, K, delta, stream)
    torch.cuda.synchronize()
    ctx.lags_profile_enable(False)
    prof2 = ctx.lags_profile_read()
    ctx.lags_profile_reset()
    delta_host = delta.cpu().numpy().reshape(-1, 3)
    ctx.lags_sparsify_model(table_b, grad, res, wl.lr, idx, val, stream)
    routes = ctx.lags_last_routes(table_b)
    route_names = {0: "one_workgroup", 1: "sampled_single_pass", 2: "sampled_fell_back", 3: "multi_pass"}
    route_elems = {}
    for (off, d, r), code in zip(batched, routes):
        route_elems[route_names[code]] = route_elems.get(route_names[code], 0) + d

    # Eq. 9 (Section 5) on a SYNTHETIC timing table: backpropagation time proportional to the layer
    # size (2.8 ns per parameter, the paper's 0.391 s for its VGG-16), the sparsification overhead
    # from this run's own rate, a 10 Gb/s network with 50 us start-up, P workers, c_u = 1000
    ds = [d for (_, d, _) in layers]
    per_elem_s = (t1 - t0) / args.steps / float(P * total)
    t_comp = [2.8e-9 * d for d in ds]
    t_spar = [per_elem_s * d for d in ds]
    ta = time.perf_counter()
    ada_k, _ = lags.lags_adaptive_ratios(50e-6, 0.8e-9, P, ds, t_comp, t_spar, 1000.0)
    ada_us = (time.perf_counter() - ta) * 1e6
    ada_c = [d / k for d, k in zip(ds, ada_k)]

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    elements = P * total
    value = elements / (ms_per_step * 1e-3)

    # dominant kernel = largest total time; its algorithmic bytes per launch
    rho_mean = float(K) / float(total)
    # elements each kernel covers in one step (per-worker mode: P calls over one worker's table)
    if args.per_worker:
        kel = {k: v * P for k, v in table_1.kernel_elements().items()}
    else:
        kel = dict(table_b.kernel_elements())
    kel.update({k: v for k, v in table_1.kernel_elements().items() if k == "k_merge"})
    dom_ms = prof[dom][0] / prof[dom][1]                 # average duration of one launch
    launches_per_step = prof[dom][1] / args.steps
    dom_ms_per_step = prof[dom][0] / args.steps
    if dom == "k_merge":
        bpe = 4.0 + 8.0 * P * rho_mean
    else:
        bpe = 12.0 + 8.0 * rho_mean
    # algorithmic bytes of the elements the kernel covers in one step / its time in one step
    # (= bytes per launch / average launch duration when every launch covers an equal share)
    achieved = bpe * kel.get(dom, elements) / (dom_ms_per_step * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": (lambda t: None if t is None else t / launches_per_step)(
                    None if args.per_worker else measured_traffic(dom, wl.name, P)),
                "avg_kernel_ms": round(dom_ms, 4), "launches_per_step": launches_per_step,
                "bytes_per_element": round(bpe, 4),
                "elements_per_launch": kel.get(dom, elements) / launches_per_step}
    kernels = {k: {"ms_per_step": round(v[0] / n_table, 4), "launches_per_step": v[1] / n_table}
               for k, v in sorted(prof_all.items(), key=lambda kv: -kv[1][0])}
    merge_names = ("k_merge", "k_merge_bounds")
    sparsify_ms = call_ms
    merge_ms = sum(prof_all.get(k, (0.0, 0))[0] for k in merge_names) / n_table

    # the practical ceiling beside the spec-sheet peak: a plain device copy of one worker's array
    ca = torch.empty(total, dtype=torch.float32, device=dev).normal_()
    cb = torch.empty_like(ca)
    for _ in range(2):
        cb.copy_(ca)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        cb.copy_(ca)
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 10 * 8.0 * total / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del ca, cb
    traffic = roofline["traffic"]
    measured_gbs = None if traffic is None else traffic / (dom_ms * 1e-3) / 1e9

    out = {
        "metric": "sparsified elements/s, per-layer top-k + error feedback (P workers) + merge",
        "value": value, "unit": "elements/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "layers": len(layers), "elements_per_worker": total, "workers": P,
                   "calls_per_step": "one sparsify call per worker + merge" if args.per_worker
                   else "one batched sparsify call (P x L layers) + merge",
                   "sum_k_per_worker": K, "lr": wl.lr, "distribution": wl.dist},
        "algorithmic_gbs": {"sparsify": round((12.0 + 8.0 * rho_mean) * elements / (sparsify_ms * 1e-3) / 1e9, 1)
                            if sparsify_ms > 0 else None,
                            "merge": round((4.0 + 8.0 * P * rho_mean) * total / (merge_ms * 1e-3) / 1e9, 1)
                            if merge_ms > 0 else None,
                            "sparsify_frac_of_peak": round((12.0 + 8.0 * rho_mean) * elements /
                                                           (sparsify_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
                            if sparsify_ms > 0 else None},
        "sparsify_call_ms": round(call_ms, 4),
        "sparsify_elements_per_s": round(elements / (call_ms * 1e-3), 1) if call_ms > 0 else None,
        "merge": {"ms": round(merge_ms, 4),
                  "update_elements_per_s": round(total / (merge_ms * 1e-3), 1) if merge_ms > 0 else None,
                  "algorithmic_gbs": round((4.0 + 8.0 * P * rho_mean) * total / (merge_ms * 1e-3) / 1e9, 1)
                  if merge_ms > 0 else None},
        "hbm": {"peak_gbs": HBM_PEAK_GBS, "plain_copy_gbs": round(copy_gbs, 1),
                "dominant_kernel_algorithmic_gbs": roofline["achieved"],
                "dominant_kernel_measured_gbs": None if measured_gbs is None else round(measured_gbs, 1),
                "dominant_kernel_measured_frac_of_peak": None if measured_gbs is None
                else round(measured_gbs / HBM_PEAK_GBS, 4),
                "dominant_kernel_frac_of_plain_copy": round(roofline["achieved"] / copy_gbs, 4)},
        "kernels": kernels,
        "elements_by_route": route_elems,
        "roofline": roofline,
        "next_rows": {
            "sparse_apply_ms": round((prof2["k_merge<apply>"][0] + prof2["k_merge_bounds"][0] / 2) / reps, 4),
            "delta_monitor_ms": round((prof2["k_delta_tiles"][0] + prof2["k_delta_finish"][0]
                                       + prof2["k_merge_bounds"][0] / 2) / reps, 4),
            "delta_monitor_gbs": round(4.0 * P * total / (prof2["k_delta_tiles"][0] / reps * 1e-3) / 1e9, 1),
            "delta_max": float(np.nanmax(delta_host[:, 2])),
            "adaptive_ratio": {"timing_table": "synthetic", "solver_us": round(ada_us, 1),
                               "layers_at_cap": sum(1 for c in ada_c if c >= 999.0),
                               "layers_below_cap": sum(1 for c in ada_c if c < 999.0),
                               "min_ratio": round(min(ada_c), 2)},
        },
    }
    if not args.no_cpu_baseline:
        threads = min(16, os.cpu_count() or 1)
        v, dt = cpu_baseline(wl, grad0_host, threads)
        extras = cpu_baseline_extras(wl, grad0_host, idx.cpu().numpy(), val.cpu().numpy(), P, K)
        out["cpu_baseline"] = {**extras, "value": v, "unit": "elements/s", "cores": threads, "kind": "oracle",
                               "sample": "worker 0 of %d, one iteration, all %d layers (%d elements), "
                                         "%.1f s wall" % (P, len(layers), total, dt)}
    print(json.dumps(out))
    table_b.destroy()
    table_1.destroy()
    ctx.destroy()


if __name__ == "__main__":
    main()
