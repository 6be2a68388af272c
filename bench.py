#!/usr/bin/env python3
"""Benchmark of the LAGS-SGD hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic gradients that are
already resident in HBM: the per-layer error-compensated top-k sparsifier for all P
workers of the workload (one batched lags_sparsify_model call over P x L layers) and
the merge of the P sparse sets into the dense averaged update (lags_merge_sparse).
The steps cycle through three pre-generated gradient iterations; the residuals carry over.

Prints ONE JSON line: sparsified elements/s (whole job) on the headline workload, the roofline
of the dominant kernel from HIP-event timings taken inside the timed region, the same figures
for all five benchmark configurations and for the call shapes a single worker would issue
(`configs`), the practical bandwidth ceiling from plain kernels of the same shape (`hbm`), and
the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak
N_ITERS = 3             # pre-generated gradient iterations that the steps cycle through


def committed_traffic(kernel, workload, workers):
    """HBM bytes per launch of `kernel` for this workload from a committed rocprofv3 counter
    summary (profiles/*.txt, lines 'FETCH_BYTES_PER_LAUNCH <kernel> <workload> P=<workers>: <bytes>'
    and 'WRITE_BYTES_PER_LAUNCH ...'): (read bytes, written bytes, file), each None where no
    summary holds it."""
    import glob
    found = {"FETCH": None, "WRITE": None}
    src = None
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        for line in open(path):
            for what in found:
                if line.startswith("%s_BYTES_PER_LAUNCH %s %s P=%d:" % (what, kernel, workload, workers)):
                    found[what] = float(line.split(":")[1])
                    src = os.path.relpath(path, ROOT)
    return found["FETCH"], found["WRITE"], src


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


class Job:
    """One workload resident in device memory: tables, gradients of N_ITERS iterations, residuals,
    outputs.  The big arrays are views of pools that the caller owns and reuses."""

    def __init__(self, torch, lags, workloads, ctx, wl, P, grad_pool, res_pool, dev):
        self.torch, self.ctx, self.wl, self.P = torch, ctx, wl, P
        total = wl.total_d
        self.total = total
        self.layers = wl.layers()
        self.batched = [(p * total + off, d, r) for p in range(P) for (off, d, r) in self.layers]
        self.table_b = ctx.table(self.batched)      # P x L layers: one sparsify call per step
        self.table_1 = ctx.table(self.layers)       # one worker's layout: the merge, per-worker calls
        self.K = self.table_1.total_k
        assert self.table_b.total_k == P * self.K
        self.grads = [grad_pool[it * P * total:(it + 1) * P * total] for it in range(N_ITERS)]
        for it in range(N_ITERS):
            for p in range(P):
                workloads.grad_torch(wl, it, p, dev, out=self.grads[it][p * total:(p + 1) * total])
        self.res = res_pool[:P * total]
        self.res.zero_()
        self.idx = torch.empty(P * self.K, dtype=torch.int32, device=dev)
        self.val = torch.empty(P * self.K, dtype=torch.float32, device=dev)
        self.upd = torch.empty(total, dtype=torch.float32, device=dev)
        self.stream = torch.cuda.current_stream()
        self.n_steps = 0
        self.rho_mean = float(self.K) / float(total)

    def sparsify(self, per_worker=False):
        g, P, total, K = self.grads[self.n_steps % N_ITERS], self.P, self.total, self.K
        if per_worker:
            for p in range(P):
                self.ctx.lags_sparsify_model(self.table_1, g[p * total:(p + 1) * total],
                                             self.res[p * total:(p + 1) * total], self.wl.lr,
                                             self.idx[p * K:(p + 1) * K], self.val[p * K:(p + 1) * K], self.stream)
        else:
            self.ctx.lags_sparsify_model(self.table_b, g, self.res, self.wl.lr, self.idx, self.val, self.stream)

    def merge(self):
        self.ctx.lags_merge_sparse(self.table_1, self.idx, self.val, self.P, self.K, self.upd, self.stream)

    def step(self, per_worker=False):
        self.sparsify(per_worker)
        self.merge()
        self.n_steps += 1

    def timed_steps(self, n, per_worker=False):
        """n steps with three events each on the stream the kernels run on: the medians of the
        sparsify call(s), the merge and the whole step in milliseconds."""
        t = self.torch
        ev = [[t.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n)]
        for i in range(n):
            ev[i][0].record(self.stream)
            self.sparsify(per_worker)
            ev[i][1].record(self.stream)
            self.merge()
            ev[i][2].record(self.stream)
            self.n_steps += 1
        t.cuda.synchronize()
        sp = statistics.median(e[0].elapsed_time(e[1]) for e in ev)
        mg = statistics.median(e[1].elapsed_time(e[2]) for e in ev)
        st = statistics.median(e[0].elapsed_time(e[2]) for e in ev)
        return sp, mg, st

    def summary(self, sp, mg, st):
        elements = self.P * self.total
        bpe_s, bpe_m = 12.0 + 8.0 * self.rho_mean, 4.0 + 8.0 * self.P * self.rho_mean
        return {"ms_per_step": round(st, 4), "elements_per_s": round(elements / (st * 1e-3), 1),
                "sparsify_ms": round(sp, 4), "merge_ms": round(mg, 4),
                "sparsify_algorithmic_gbs": round(bpe_s * elements / (sp * 1e-3) / 1e9, 1),
                "sparsify_frac_of_peak": round(bpe_s * elements / (sp * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                "merge_algorithmic_gbs": round(bpe_m * self.total / (mg * 1e-3) / 1e9, 1)}

    def routes(self):
        names = {0: "one_workgroup", 1: "sampled_single_pass", 2: "sampled_fell_back", 3: "multi_pass"}
        self.ctx.lags_sparsify_model(self.table_b, self.grads[self.n_steps % N_ITERS], self.res, self.wl.lr,
                                     self.idx, self.val, self.stream)
        self.n_steps += 1
        out = {}
        for (off, d, r), code in zip(self.batched, self.ctx.lags_last_routes(self.table_b)):
            out[names[code]] = out.get(names[code], 0) + d
        return out

    def close(self):
        self.table_b.destroy()
        self.table_1.destroy()


def layer_sweep(torch, lags, job, reps=10):
    """One lags_sparsify_layer call per layer of worker 0 (the call shape of a worker that
    sparsifies every layer as soon as its gradient exists): microseconds per call, calls back to back."""
    ctx, wl = job.ctx, job.wl
    g_all, r_all = job.grads[0][:job.total], job.res[:job.total]
    rows, total_us = [], 0.0
    for (off, d, rho) in job.layers:
        k = lags.lags_topk_count(d, rho)
        g, r = g_all[off:off + d], r_all[off:off + d]
        oi, ov = job.idx[:k], job.val[:k]
        for _ in range(2):
            ctx.lags_sparsify_layer(g, r, wl.lr, k, oi, ov, job.stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(job.stream)
        for _ in range(reps):
            ctx.lags_sparsify_layer(g, r, wl.lr, k, oi, ov, job.stream)
        e1.record(job.stream)
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / reps * 1e3
        total_us += us
        rows.append((d, us))
    rows.sort(key=lambda t: -t[0])
    bytes_alg = (12.0 + 8.0 * job.rho_mean) * job.total
    return {"calls": len(rows), "sum_us": round(total_us, 1),
            "algorithmic_frac_of_peak": round(bytes_alg / (total_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
            "largest_layers_us": [{"d": d, "us": round(us, 1)} for d, us in rows[:4]],
            "median_us": round(statistics.median(us for _, us in rows), 1)}


def graph_step_ms(torch, lags, workloads, w, grad_pool, res_pool, dev, reps=50):
    """One step (batched sparsify + merge) of a small table recorded into a HIP graph, in a context
    of its own after warm-up calls have sized its scratch, and replayed back to back: milliseconds
    per replay.  The recorded step reads the first gradient iteration every time; the residuals evolve."""
    ctx = lags.Context(0)
    j = Job(torch, lags, workloads, ctx, w, w.P, grad_pool, res_pool, dev)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        j.stream = side
        j.step()
        j.step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        j.stream = torch.cuda.current_stream()
        j.n_steps = 0
        j.step()
    torch.cuda.synchronize()
    for _ in range(3):
        graph.replay()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    del graph
    j.close()
    ctx.destroy()
    return ms


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="vgg16", help="single|resnet20|vgg16|resnet50|lstm|inception4")
    ap.add_argument("--rho", default="0.001", help="density for every layer, or 'config' for the workload's own")
    ap.add_argument("--workers", type=int, default=0, help="simulated workers P (0 = the workload's)")
    ap.add_argument("--per-worker", action="store_true",
                    help="one lags_sparsify_model call per worker (L layers each) instead of one batched call")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the block of the other configurations")
    ap.add_argument("--progress", action="store_true", help="name every stage on stderr as it starts")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of 1 GiB (for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path has no inter-GPU step); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    def stage(name):
        if args.progress:
            print("bench.py: " + name, file=sys.stderr, flush=True)

    stage("import torch")
    import numpy as np
    import torch
    from paper_1911_08727_amd import hbmcal, lags, workloads

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
    # every job of this run lives in these two pools (sized for the largest one)
    other = [] if args.no_configs else [workloads.make(n) for n in workloads.NAMES + workloads.EXTRA_NAMES]
    pool_elems = max([P * wl.total_d] + [w.P * w.total_d for w in other])
    grad_pool = torch.empty(N_ITERS * pool_elems, dtype=torch.float32, device=dev)
    res_pool = torch.empty(pool_elems, dtype=torch.float32, device=dev)

    stage("tables and synthetic gradients")
    ctx = lags.Context(0)
    job = Job(torch, lags, workloads, ctx, wl, P, grad_pool, res_pool, dev)
    total, K, layers = job.total, job.K, job.layers
    grad0_host = None if args.no_cpu_baseline else job.grads[0][:total].cpu().numpy()

    stage("warm-up steps")
    for _ in range(args.warmup):
        job.step(args.per_worker)
    torch.cuda.synchronize()
    # an untimed pass with every kernel bracketed by events: the per-kernel table, and which
    # kernel dominates
    stage("per-kernel pass")
    ctx.lags_profile_reset()
    ctx.lags_profile_enable(True)
    n_table = max(2, min(5, args.steps))
    for _ in range(n_table):
        job.step(args.per_worker)
    torch.cuda.synchronize()
    ctx.lags_profile_enable(False)
    prof_all = ctx.lags_profile_read()
    ctx.lags_profile_reset()
    prof_all.pop("sparsify_call", None)
    dom = max(prof_all, key=lambda k: prof_all[k][0])
    # the timed region: exactly K steps; only the dominant kernel is bracketed by HIP events
    # (on the stream it is launched on), so the measurement adds two events per step
    stage("timed steps")
    ctx.lags_profile_enable_kernel(dom)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        job.step(args.per_worker)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ctx.lags_profile_enable(False)
    prof = ctx.lags_profile_read()
    ctx.lags_profile_reset()
    # the two calls of a step apart, two events each (no per-kernel events)
    stage("steps with one event pair per call")
    sp_ms, mg_ms, st_ms = job.timed_steps(max(3, min(10, args.steps)), args.per_worker)
    headline = job.summary(sp_ms, mg_ms, st_ms)

    # the rows next to the hot path, measured apart from the timed steps: the in-place sparse
    # parameter step (Algorithm 1 line 9) and the delta metric of Section 6.2
    stage("sparse apply and delta metric")
    param = torch.zeros(total, dtype=torch.float32, device=dev)
    delta = torch.empty(3 * len(layers), dtype=torch.float64, device=dev)
    reps = 5
    stream = job.stream
    ctx.lags_apply_sparse(job.table_1, job.idx, job.val, P, K, param, stream)
    ctx.lags_delta_monitor(job.table_1, job.res, total, job.idx, job.val, P, K, delta, stream)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2 * reps + 1)]
    ev[0].record(stream)
    for i in range(reps):
        ctx.lags_apply_sparse(job.table_1, job.idx, job.val, P, K, param, stream)
        ev[2 * i + 1].record(stream)
        ctx.lags_delta_monitor(job.table_1, job.res, total, job.idx, job.val, P, K, delta, stream)
        ev[2 * i + 2].record(stream)
    torch.cuda.synchronize()
    apply_ms = statistics.median(ev[2 * i].elapsed_time(ev[2 * i + 1]) for i in range(reps))
    delta_ms = statistics.median(ev[2 * i + 1].elapsed_time(ev[2 * i + 2]) for i in range(reps))
    delta_host = delta.cpu().numpy().reshape(-1, 3)
    stage("routes")
    route_elems = job.routes()

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
    rho_mean = job.rho_mean
    if args.per_worker:
        kel = {k: v * P for k, v in job.table_1.kernel_elements().items()}
    else:
        kel = dict(job.table_b.kernel_elements())
    kel.update({k: v for k, v in job.table_1.kernel_elements().items() if k == "k_merge"})
    dom_ms = prof[dom][0] / prof[dom][1]                 # average duration of one launch
    launches_per_step = prof[dom][1] / args.steps
    dom_ms_per_step = prof[dom][0] / args.steps
    bpe = 4.0 + 8.0 * P * rho_mean if dom == "k_merge" else 12.0 + 8.0 * rho_mean
    # algorithmic bytes of the elements the kernel covers in one step / its time in one step
    # (= bytes per launch / average launch duration when every launch covers an equal share)
    achieved = bpe * kel.get(dom, elements) / (dom_ms_per_step * 1e-3) / 1e9
    # HBM bytes per launch from the committed counter summary; `traffic` needs both counters
    t_fetch, t_write, traffic_file = (None, None, None) if args.per_worker else committed_traffic(dom, wl.name, P)
    traffic = None if t_fetch is None or t_write is None else t_fetch + t_write
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic,
                "traffic_fetch": t_fetch, "traffic_write": t_write,
                "traffic_source": None if traffic_file is None else
                "%s (rocprofv3 --pmc runs committed with the tree, not measured in this run; "
                "a counter that is null there was not collected)" % traffic_file,
                "avg_kernel_ms": round(dom_ms, 4), "launches_per_step": launches_per_step,
                "bytes_per_element": round(bpe, 4),
                "elements_per_launch": kel.get(dom, elements) / launches_per_step}
    kernels = {k: {"ms_per_step": round(v[0] / n_table, 4), "launches_per_step": v[1] / n_table}
               for k, v in sorted(prof_all.items(), key=lambda kv: -kv[1][0])}

    # the practical ceiling beside the data sheet's peak: plain kernels of the streaming pass's
    # shape (libhbmcal.so) on an array the size of the largest layer and on one as large as all
    # workers' arrays; with and without the streaming pass's occupancy cap
    stage("plain streaming kernels")
    sink = torch.zeros(64, dtype=torch.float32, device=dev)
    big_n = (pool_elems // 4096) * 4096
    small_n = min(big_n, (102760448 // 4096) * 4096)
    cal = {}
    for label, n in (("392MiB", small_n), ("all_workers", big_n)):
        a, b = grad_pool[:n], res_pool[:n]
        cal[label] = {"elements": n}
        for kind in ("copy", "read", "triad"):
            cal[label][kind + "_gbs"] = round(hbmcal.gbs(kind, a, b, sink, n, 5 if n > (1 << 29) else 20, 40960,
                                                         stream), 1)
        cal[label]["triad_gbs_without_occupancy_cap"] = round(
            hbmcal.gbs("triad", a, b, sink, n, 5 if n > (1 << 29) else 20, 0, stream), 1)
    triad = cal["all_workers"]["triad_gbs"]
    job.res.zero_()   # the calibration kernels wrote into the residual pool

    out = {
        "metric": "sparsified elements/s, per-layer top-k + error feedback (P workers) + merge",
        "value": value, "unit": "elements/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "layers": len(layers), "elements_per_worker": total, "workers": P,
                   "calls_per_step": "one sparsify call per worker + merge" if args.per_worker
                   else "one batched sparsify call (P x L layers) + merge",
                   "sum_k_per_worker": K, "lr": wl.lr, "distribution": wl.dist,
                   "gradient_iterations_cycled": N_ITERS},
        "sparsify": {"ms": headline["sparsify_ms"], "elements_per_s": round(elements / (sp_ms * 1e-3), 1),
                     "algorithmic_gbs": headline["sparsify_algorithmic_gbs"],
                     "frac_of_peak": headline["sparsify_frac_of_peak"],
                     "timing": "two HIP events around the call, median of %d steps" % max(3, min(10, args.steps))},
        "merge": {"ms": headline["merge_ms"],
                  "update_elements_per_s": round(total / (mg_ms * 1e-3), 1),
                  "algorithmic_gbs": headline["merge_algorithmic_gbs"]},
        "hbm": {"peak_gbs": HBM_PEAK_GBS, "plain_kernels": cal,
                "dominant_kernel_algorithmic_gbs": roofline["achieved"],
                "dominant_kernel_frac_of_plain_triad": round(roofline["achieved"] / triad, 4),
                "dominant_kernel_read_counter_gbs_from_committed_profile":
                    None if t_fetch is None else round(t_fetch / (dom_ms * 1e-3) / 1e9, 1),
                "dominant_kernel_read_counter_over_algorithmic_read":
                    None if t_fetch is None or dom != "k_stream" else
                    round(t_fetch / (8.0 * kel.get(dom, elements) / launches_per_step), 4)},
        "kernels": kernels,
        "elements_by_route": route_elems,
        "roofline": roofline,
        "next_rows": {
            "sparse_apply_ms": round(apply_ms, 4),
            "delta_monitor_ms": round(delta_ms, 4),
            "delta_monitor_gbs": round(4.0 * P * total / (delta_ms * 1e-3) / 1e9, 1),
            "delta_max": float(np.nanmax(delta_host[:, 2])),
            "adaptive_ratio": {"timing_table": "synthetic", "solver_us": round(ada_us, 1),
                               "layers_at_cap": sum(1 for c in ada_c if c >= 999.0),
                               "layers_below_cap": sum(1 for c in ada_c if c < 999.0),
                               "min_ratio": round(min(ada_c), 2)},
        },
    }
    idx_host, val_host = job.idx.cpu().numpy(), job.val.cpu().numpy()

    if not args.no_configs:
        stage("other call shapes and configurations")
        # the call shapes a single worker would issue, on the headline workload
        configs = {}
        sp, mg, st = job.timed_steps(5, per_worker=True)
        configs["%s, one call per worker" % wl.name] = job.summary(sp, mg, st)
        configs["%s, one lags_sparsify_layer call per layer (worker 0)" % wl.name] = layer_sweep(torch, lags, job)
        job.close()
        # the five benchmark configurations (and the Inception-v4-shaped table) at their own densities, batched calls
        for w in other:
            j = Job(torch, lags, workloads, ctx, w, w.P, grad_pool, res_pool, dev)
            for _ in range(2):
                j.step()
            sp, mg, st = j.timed_steps(6)
            row = j.summary(sp, mg, st)
            row.update({"workers": w.P, "layers": len(j.layers), "elements_per_worker": j.total,
                        "sum_k_per_worker": j.K, "elements_by_route": j.routes()})
            configs["%s (config densities)" % w.name] = row
            j.close()
            if row["ms_per_step"] < 0.3:
                # a step this short is a handful of launches: what it costs without the host's launch calls
                row["graph_replay_ms_per_step"] = round(graph_step_ms(torch, lags, workloads, w, grad_pool,
                                                                      res_pool, dev), 4)
        out["configs"] = configs
    else:
        job.close()

    if not args.no_cpu_baseline:
        stage("oracle on the host cores")
        threads = min(16, os.cpu_count() or 1)
        v, dt = cpu_baseline(wl, grad0_host, threads)
        extras = cpu_baseline_extras(wl, grad0_host, idx_host, val_host, P, K)
        out["cpu_baseline"] = {**extras, "value": v, "unit": "elements/s", "cores": threads, "kind": "oracle",
                               "sample": "worker 0 of %d, one iteration, all %d layers (%d elements), "
                                         "%.1f s wall" % (P, len(layers), total, dt)}
    print(json.dumps(out))
    ctx.destroy()


if __name__ == "__main__":
    main()
