#!/usr/bin/env python3
"""Benchmark of the bi-level l1,inf projection on one MI355X.

A "step" is one whole projection (aggregate, threshold search, clip) of one matrix that is
already resident in HBM.  The headline workload is the 4096 x 4096 fp32 matrix; the timed loop
rotates through enough (Y, X) buffer pairs that the 256 MB Infinity Cache cannot serve the
first read of Y (a cold measurement).  Two JSON lines go to stdout: first everything bulky
({"detail": ...}: per-kernel intervals, the other workloads and variants, sweeps, batches; also
written to gpurun_out/bench_detail.json), then, LAST, one compact record (under 2 KB):

  value          effective GB/s = 8 bytes/element * n*m / time  (read Y once, write X once)
  ms_per_step    milliseconds per projection
  roofline       the dominant kernel against the 8 TB/s HBM peak, timed with HIP events
  cpu_baseline   the CPU oracle on the same workload on this host: one thread, and all usable
                 cores with the columns split over worker processes (Sec. 6.2's decomposition)
  other_workloads  ms and fraction of the peak for the other configurations (--quick skips)
"""
import argparse
import json
import os
import statistics
import zlib
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM-side bytes per launch of the map kernel from the rocprofv3 --pmc runs summarised in
# profiles/ (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, in KiB), valid for these library versions only.
TRAFFIC_VERSIONS = (382, 383, 384, 385, 386)   # the library versions the counters in profiles/ hold for (383, 385 and 386 changed l1,1 kernels only, 384 no kernel)
TRAFFIC_KIB = {"square_4096": 32979.1 * 1.999 + 65557.7, "square_16384": 524922.6 * 1.999 + 1048622.9,
               "tensor_256x256x256": 32906.8 * 1.999 + 65625.0}
INFINITY_CACHE_BYTES = 256 * 1024 * 1024


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="square_4096")
    ap.add_argument("--variant", default="l1inf", choices=["l1inf", "l12", "l11"],
                    help="bi-level variant timed on the workload (other than l1inf: as --quick, for profiling runs)")
    ap.add_argument("--quick", action="store_true", help="headline workload only, no CPU baseline")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU baseline")
    return ap.parse_args()


def device_eta(mp, Yd, variant, frac, ws):
    """eta = frac * ||Y||_{1,q}, the norm taken by the library on the device, rounded to fp32."""
    import numpy as np
    return float(np.float32(frac * mp.norm_l1q(Yd, variant, workspace=ws)))


def time_calls(torch, fn, pairs, steps, warmup):
    """Wall-clock ms per call over `steps` calls that rotate through `pairs`."""
    for i in range(warmup):
        fn(*pairs[i % len(pairs)])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        fn(*pairs[i % len(pairs)])
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


DIST_TEXT = {"normal": "i.i.d. N(0,1)", "normal_colscale": "N(0,1) x per-column scale log-uniform in [0.01,1]",
             "laplace": "i.i.d. Laplace(0,1)", "uniform": "i.i.d. U(0,1)"}

KERNEL_LABELS = {
    3: ["held_clear", "held_slab+search"],
    4: ["colagg", "reduce", "colmap+search"],
    5: ["colagg", "reduce", "search", "colmap"],
    6: ["colagg", "reduce", "search", "l11_sweeps", "colmap"],
}


def time_kernels(torch, mp, fn, pairs, steps, warmup):
    """Average duration (ms) of every kernel of a call, from HIP events the library records on
    the launch stream before each kernel and after the last one (mlproj_trace_*), inside the
    same rotating loop the wall-clock figure uses."""
    for i in range(warmup):
        fn(*pairs[i % len(pairs)])
    torch.cuda.synchronize()
    tr = mp.KernelTrace(steps * 8)
    with tr:
        for i in range(steps):
            fn(*pairs[i % len(pairs)])
    d = tr.durations_ms()
    per_call = tr.count // steps
    tr.close()
    labels = KERNEL_LABELS[per_call]
    out = {}
    for k, name in enumerate(labels):
        out[name] = statistics.mean(d[i * per_call + k] for i in range(steps))
    return out


def bench_bilevel(torch, mp, Y_host, variant, frac, steps, warmup, cold=True, eta_abs=None, storage="f32",
                  keep_output=False, weighted=False, outer=1):
    """storage "bf16" / "f16": the same matrix rounded to 16 bits, through bilevel_proj_stored
    (half the bytes: 4 per element instead of 8 in the effective figures).
    weighted: the weighted l1 ball as outer norm (fp32 storage), weights exp(U(-1, 1)) seeded by
    the shape, eta = frac * sum_j w_j v_j.  outer = 2 or "inf": the l2 or l_inf ball as outer norm
    (fp32 storage), eta = frac * ||v||_2 or frac * max v."""
    import numpy as np
    dev = torch.device("cuda:0")
    n, m = Y_host.shape
    elem = 4 if storage == "f32" else 2
    nbytes = n * m * elem
    npairs = 1
    if cold and 2 * nbytes < 2 * INFINITY_CACHE_BYTES:
        npairs = max(2, -(-3 * INFINITY_CACHE_BYTES // (2 * nbytes)))   # > 3 caches of working set
    Y0 = torch.from_numpy(Y_host).to(dev)
    ws = mp.Workspace.for_call(variant, n, m, device=dev)
    if storage != "f32":
        Y0 = Y0.to({"bf16": torch.bfloat16, "f16": torch.float16}[storage])
        eta = device_eta(mp, Y0.float(), variant, frac, ws) if eta_abs is None else float(eta_abs)
        q = {"l1inf": "inf", "l11": 1, "l12": 2}[variant]
        fn = lambda Y, eta, X, workspace, v_out=None: mp.bilevel_proj_stored(Y, eta, q, X=X, workspace=workspace, v_out=v_out)
    elif weighted:
        q = {"l1inf": "inf", "l11": 1, "l12": 2}[variant]
        wts = torch.from_numpy(np.exp(np.random.default_rng([n, m, 17]).uniform(-1, 1, m)).astype(np.float32)).to(dev)
        vbuf = torch.empty(m, dtype=torch.float32, device=dev)
        mp.bilevel_proj_stored(Y0, 1.0, q, workspace=ws, v_out=vbuf)      # (only for v)
        eta = float(np.float32(frac * float((wts.double() * vbuf.double()).sum().item())))
        fn = lambda Y, eta, X, workspace, v_out=None: mp.bilevel_proj_weighted(Y, eta, q, wts, X=X, workspace=workspace, v_out=v_out)
    elif outer != 1:
        q = {"l1inf": "inf", "l11": 1, "l12": 2}[variant]
        vbuf = torch.empty(m, dtype=torch.float32, device=dev)
        mp.bilevel_proj_stored(Y0, 1.0, q, workspace=ws, v_out=vbuf)      # (only for v)
        norm_p = float(vbuf.double().norm().item()) if outer == 2 else float(vbuf.max().item())
        eta = float(np.float32(frac * norm_p))
        fn = lambda Y, eta, X, workspace, v_out=None: mp.bilevel_proj_stored(Y, eta, q, p=outer, X=X, workspace=workspace, v_out=v_out)
    else:
        eta = device_eta(mp, Y0, variant, frac, ws) if eta_abs is None else float(eta_abs)
        fn = getattr(mp, "bilevel_proj_" + variant)
    pairs = [(Y0, torch.empty_like(Y0))] + [(Y0.clone(), torch.empty_like(Y0)) for _ in range(npairs - 1)]
    ms = time_calls(torch, lambda Y, X: fn(Y, eta, X=X, workspace=ws), pairs, steps, warmup)
    res = ws.result()
    x_timed = pairs[(steps - 1) % npairs][1].cpu().numpy() if keep_output else None   # X of the last timed step
    # how far the nearest aggregate is from the threshold, relative: the support is safe
    # against fp64 summation-order differences as long as this is far above 1e-13
    vbuf = torch.empty(m, dtype=torch.float32, device=dev)
    fn(pairs[0][0], eta, X=pairs[0][1], workspace=ws, v_out=vbuf)
    ratio = vbuf.double() / wts.double() if weighted else vbuf.double()    # column j is kept when v_j / w_j > tau
    margin = float(((ratio - res["tau"]).abs().min() / res["tau"]).item()) if res["tau"] > 0 else None
    k_raw = time_kernels(torch, mp, lambda Y, X: fn(Y, eta, X=X, workspace=ws), pairs, min(steps, 100), min(warmup, 10))
    # Bracketing every kernel with events drains the queue around it, which adds the same
    # dispatch-from-idle latency to every interval; the untraced loop above has none of it.
    # Spread the difference evenly: interval - (sum of intervals - untraced ms per call) / kernels.
    excess = max(0.0, (sum(k_raw.values()) - ms) / len(k_raw))
    k_ms = {k: max(v - excess, 0.0) for k, v in k_raw.items()}
    warm_ms = time_calls(torch, lambda Y, X: fn(Y, eta, X=X, workspace=ws), pairs[:1], steps, warmup) if npairs > 1 else ms
    # spread of the cold figure: ten more loops of steps/10 calls each
    chunk = max(1, steps // 10)
    chunks = [time_calls(torch, lambda Y, X: fn(Y, eta, X=X, workspace=ws), pairs, chunk, 0) for _ in range(10)]
    elems = n * m
    b = 2.0 * elem   # read Y once, write X once
    out = {
        "shape": [n, m], "variant": variant, "storage": storage, "eta": eta, "buffer_pairs": npairs,
        "ms": ms, "ms_warm": warm_ms,
        "ms_median_of_10_chunks": statistics.median(chunks), "ms_min_of_10_chunks": min(chunks),
        "bytes_per_element_rw": b,   # "rw": read Y once + write X once; "rrw": two reads + one write
        "eff_GBps_rw": b * elems / ms / 1e6,
        "frac_of_peak_rw": b * elems / ms / 1e6 / HBM_PEAK_GBS,
        "eff_GBps_rrw": 1.5 * b * elems / ms / 1e6,
        "kernel_ms": k_ms, "kernel_ms_event_intervals": k_raw,
        "tau": res["tau"], "n_active": res["n_active"], "support_margin": margin,
        "search_iters": res["search_iters"],
        "inner_sweeps": res["inner_sweeps"], "inner_pending": res["inner_pending"],
    }
    if keep_output:
        out["_x_timed"] = x_timed
    del pairs
    torch.cuda.empty_cache()
    return out


def bench_trilevel_head(torch, mp, Y_host, frac, steps, warmup, keep_output=False):
    """The tri-level l1,inf,inf projection as the headline workload (--workload tensor_...): the
    fields bench_bilevel reports, cold timing over rotating buffers."""
    import numpy as np
    dev = torch.device("cuda:0")
    d0 = Y_host.shape[0]
    npairs = max(2, -(-3 * INFINITY_CACHE_BYTES // (2 * Y_host.nbytes)))
    Y0 = torch.from_numpy(Y_host).to(dev)
    pairs = [(Y0, torch.empty_like(Y0))] + [(Y0.clone(), torch.empty_like(Y0)) for _ in range(npairs - 1)]
    ws = mp.Workspace.for_call("tri", *Y_host.shape, device=dev)
    # eta from the library itself: with a radius beyond the norm the record holds the norm
    mp.trilevel_proj_l1infinf(pairs[0][0], 3.0e38, X=pairs[0][1], workspace=ws)
    torch.cuda.synchronize()
    eta = float(np.float32(frac * ws.result()["norm"]))
    fn = lambda Y, X: mp.trilevel_proj_l1infinf(Y, eta, X=X, workspace=ws)
    ms = time_calls(torch, fn, pairs, steps, warmup)
    res = ws.result()
    x_timed = pairs[(steps - 1) % npairs][1].cpu().numpy() if keep_output else None
    k_raw = time_kernels(torch, mp, fn, pairs, min(steps, 100), min(warmup, 10))
    excess = max(0.0, (sum(k_raw.values()) - ms) / len(k_raw))
    k_ms = {k: max(v - excess, 0.0) for k, v in k_raw.items()}
    warm_ms = time_calls(torch, fn, pairs[:1], steps, warmup)
    elems = Y_host.size
    out = {"shape": list(Y_host.shape), "variant": "tri", "storage": "f32", "eta": eta, "buffer_pairs": npairs,
           "ms": ms, "ms_warm": warm_ms, "bytes_per_element_rw": 8.0, "eff_GBps_rw": 8.0 * elems / ms / 1e6,
           "frac_of_peak_rw": 8.0 * elems / ms / 1e6 / HBM_PEAK_GBS, "kernel_ms": k_ms,
           "kernel_ms_event_intervals": k_raw, "tau": res["tau"], "n_active": res["n_active"],
           "search_iters": res["search_iters"]}
    if keep_output:
        out["_x_timed"] = x_timed
    del pairs
    torch.cuda.empty_cache()
    return out


def bench_tensor(torch, mp, Y_host, frac, steps, warmup):
    """Tri-level l1,inf,inf (its own entry point) and the generic multi-level engine on a 3-D tensor."""
    import numpy as np
    dev = torch.device("cuda:0")
    d0 = Y_host.shape[0]
    npairs = max(2, -(-3 * INFINITY_CACHE_BYTES // (2 * Y_host.nbytes)))
    Y0 = torch.from_numpy(Y_host).to(dev)
    pairs = [(Y0, torch.empty_like(Y0))] + [(Y0.clone(), torch.empty_like(Y0)) for _ in range(npairs - 1)]
    elems = Y_host.size
    out = {}

    def record(name, fn, ws, eta):
        ms = time_calls(torch, fn, pairs, steps, warmup)
        res = ws.result()
        out[name] = {"shape": list(Y_host.shape), "eta": eta, "ms": ms, "eff_GBps_rw": 8.0 * elems / ms / 1e6,
                     "frac_of_peak_rw": 8.0 * elems / ms / 1e6 / HBM_PEAK_GBS, "tau": res["tau"],
                     "n_active": res["n_active"]}

    # eta from the library itself: the nested norm is the sum of the aggregate vector
    for name, norms in (("l1infinf", ["inf", "inf"]), ("l111", [1, 1]), ("l122", [2, 2])):
        ws = mp.Workspace(mp.multilevel_workspace_bytes(Y_host.shape), device=dev)
        v = torch.empty(d0, dtype=torch.float32, device=dev)
        mp.multilevel_proj(pairs[0][0], norms, 3.0e38, X=pairs[0][1], workspace=ws, v_out=v)
        torch.cuda.synchronize()
        eta = float(np.float32(frac * ws.result()["norm"]))
        if name == "l1infinf":
            ws3 = mp.Workspace.for_call("tri", *Y_host.shape, device=dev)
            record("trilevel_proj_l1infinf", lambda Y, X: mp.trilevel_proj_l1infinf(Y, eta, X=X, workspace=ws3), ws3, eta)
        record("multilevel_proj/" + name, lambda Y, X: mp.multilevel_proj(Y, norms, eta, X=X, workspace=ws), ws, eta)
        if name == "l111":
            # the weighted l1 ball on top: weights exp(U(-1, 1)) seeded by the shape, eta = frac * sum_a w_a v_a
            wts = torch.from_numpy(np.exp(np.random.default_rng(list(Y_host.shape) + [17]).uniform(-1, 1, d0)).astype(np.float32)).to(dev)
            eta_w = float(np.float32(frac * float((wts.double() * v.double()).sum().item())))
            record("multilevel_proj_weighted/" + name,
                   lambda Y, X: mp.multilevel_proj_weighted(Y, norms, eta_w, wts, X=X, workspace=ws), ws, eta_w)
    # the same tensor stored in bf16 (4 bytes per element moved instead of 8)
    del pairs
    torch.cuda.empty_cache()
    Yb = Y0.to(torch.bfloat16)
    pairs = [(Yb, torch.empty_like(Yb))] + [(Yb.clone(), torch.empty_like(Yb)) for _ in range(2 * npairs - 1)]
    for name, norms in (("l111", [1, 1]),):
        ws = mp.Workspace(mp.multilevel_workspace_bytes(Y_host.shape), device=dev)
        mp.multilevel_proj_stored(pairs[0][0], norms, 3.0e38, X=pairs[0][1], workspace=ws)
        torch.cuda.synchronize()
        eta = float(np.float32(frac * ws.result()["norm"]))
        record("multilevel_proj_stored/" + name + "/bf16",
               lambda Y, X: mp.multilevel_proj_stored(Y, norms, eta, X=X, workspace=ws), ws, eta)
        out["multilevel_proj_stored/" + name + "/bf16"]["eff_GBps_rw"] /= 2
        out["multilevel_proj_stored/" + name + "/bf16"]["frac_of_peak_rw"] /= 2
    del pairs
    torch.cuda.empty_cache()
    return out


def linear_fit(sizes, times_ms):
    """Least squares time = a + b * elements: (a in us, b in ns per 1000 elements, R^2)."""
    import numpy as np
    x, y = np.asarray(sizes, dtype=np.float64), np.asarray(times_ms, dtype=np.float64) * 1e3
    b, a = np.polyfit(x, y, 1)
    r2 = 1.0 - float(((y - (a + b * x)) ** 2).sum() / ((y - y.mean()) ** 2).sum())
    return {"intercept_us": float(a), "ns_per_1000_elements": float(b) * 1e6, "r2": r2}


def bench_size_sweep(torch, mp, workloads, steps, warmup):
    """The size sweeps of the paper's timing figures (Sec. 6.1) on U(0,1) entries: the bi-level
    l1,inf projection at eta = 1 with 1000 columns and a growing number of rows, with 1000 rows and
    a growing number of columns, and the tri-level l1,inf,inf and l1,1,1 projections of a tensor
    of 32 channels x 1000 x m (here C-order (m, 1000, 32): groups on the first axis, the channel
    axis innermost), eta = 0.2 * norm.  Cold timing (rotating buffers), with a straight-line fit."""
    import numpy as np
    dev = torch.device("cuda:0")
    out = {}
    for key, shapes in (("bilevel_l1inf/rows_x_1000", [(k * 1000, 1000) for k in (1, 2, 4, 8, 16, 32)]),
                        ("bilevel_l1inf/1000_x_columns", [(1000, k * 1000) for k in (1, 2, 4, 8, 16, 32)])):
        rows = []
        for i, shape in enumerate(shapes):
            Y = workloads.generate(shape, "uniform", workloads.BASE_SEED + 100 + i)
            Y0 = torch.from_numpy(Y).to(dev)
            npairs = max(2, -(-3 * INFINITY_CACHE_BYTES // (2 * Y.nbytes)))
            pairs = [(Y0, torch.empty_like(Y0))] + [(Y0.clone(), torch.empty_like(Y0)) for _ in range(npairs - 1)]
            ws = mp.Workspace.for_call("l1inf", shape[0], shape[1], device=dev)
            ms = time_calls(torch, lambda Yd, Xd: mp.bilevel_proj_l1inf(Yd, 1.0, X=Xd, workspace=ws), pairs, steps, warmup)
            rows.append({"shape": list(shape), "ms": ms, "n_active": ws.result()["n_active"]})
            del pairs, Y0
            torch.cuda.empty_cache()
        out[key] = {"eta": 1.0, "rows": rows,
                    "fit": linear_fit([r["shape"][0] * r["shape"][1] for r in rows], [r["ms"] for r in rows])}
    for name, norms in (("l1infinf", ["inf", "inf"]), ("l111", [1, 1])):
        rows = []
        for i, m in enumerate((250, 500, 1000, 2000)):
            shape = (m, 1000, 32)
            Y = workloads.generate(shape, "uniform", workloads.BASE_SEED + 200 + i)
            Y0 = torch.from_numpy(Y).to(dev)
            npairs = max(2, -(-3 * INFINITY_CACHE_BYTES // (2 * Y.nbytes)))
            pairs = [(Y0, torch.empty_like(Y0))] + [(Y0.clone(), torch.empty_like(Y0)) for _ in range(npairs - 1)]
            ws = mp.Workspace(mp.multilevel_workspace_bytes(shape), device=dev)
            mp.multilevel_proj(pairs[0][0], norms, 3.0e38, X=pairs[0][1], workspace=ws)
            torch.cuda.synchronize()
            eta = float(np.float32(0.2 * ws.result()["norm"]))
            ms = time_calls(torch, lambda Yd, Xd: mp.multilevel_proj(Yd, norms, eta, X=Xd, workspace=ws), pairs, steps, warmup)
            rows.append({"shape": list(shape), "eta": eta, "ms": ms, "n_active": ws.result()["n_active"]})
            del pairs, Y0
            torch.cuda.empty_cache()
        out["trilevel_" + name + "/m_x_1000_x_32"] = {
            "rows": rows, "fit": linear_fit([r["shape"][0] * 32000 for r in rows], [r["ms"] for r in rows])}
    return out


def bench_small(torch, mp, Y_host, frac, steps, warmup):
    """The small workload is launch-bound: eager calls (out of place, and in place as a training
    loop calls it) against replays of one call captured in a HIP graph."""
    dev = torch.device("cuda:0")
    n, m = Y_host.shape
    Y = torch.from_numpy(Y_host).to(dev)
    X = torch.empty_like(Y)
    ws = mp.Workspace.for_call("l1inf", n, m, device=dev)
    eta = device_eta(mp, Y, "l1inf", frac, ws)
    call = lambda: mp.bilevel_proj_l1inf(Y, eta, X=X, workspace=ws)
    call()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    # in place, as a training loop calls it: a fresh copy of Y for every call (a projected matrix
    # lies in the ball already, and projecting it again would be less work)
    fresh = iter([Y.clone() for _ in range(steps + warmup)])
    def in_place():
        Z = next(fresh)
        mp.bilevel_proj_l1inf(Z, eta, X=Z, workspace=ws)
    out = {"shape": [n, m]}
    for name, fn in (("ms_eager", call), ("ms_eager_in_place", in_place), ("ms_graph_replay", graph.replay)):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        out[name] = (time.perf_counter() - t0) * 1e3 / steps
    return out


def bench_batch(torch, mp, shape, count, frac, steps, warmup, variant="l1inf"):
    """`count` matrices of one shape: one bilevel_proj_batch call against a loop of single calls."""
    import numpy as np
    from paper_2405_02086_amd import workloads
    dev = torch.device("cuda:0")
    Ys = [torch.from_numpy(workloads.generate(shape, "normal", workloads.BASE_SEED + 100 + i)).to(dev) for i in range(count)]
    Xs = [torch.empty_like(Y) for Y in Ys]
    wss = [mp.Workspace.for_call(variant, shape[0], shape[1], device=dev) for _ in Ys]
    etas = [device_eta(mp, Y, variant, frac, ws) for Y, ws in zip(Ys, wss)]
    single = getattr(mp, "bilevel_proj_" + variant)
    q = {"l1inf": "inf", "l11": 1, "l12": 2}[variant]

    def loop():
        for Y, X, ws, eta in zip(Ys, Xs, wss, etas):
            single(Y, eta, X=X, workspace=ws)

    def batch():
        mp.bilevel_proj_batch(Ys, etas, q, Xs=Xs, workspaces=wss)

    prepared = mp.PreparedBatch(Ys, etas, q, Xs=Xs, workspaces=wss)   # argument block marshalled once
    # X = Y, as a training loop projects: fresh copies for every call (a projected matrix lies in the
    # ball already, and projecting it again would be less work)
    def one_in_place():
        Zs = [Y.clone() for Y in Ys]
        return mp.PreparedBatch(Zs, etas, q, Xs=Zs, workspaces=wss)
    fresh = iter([one_in_place() for _ in range(steps + warmup)])
    prepared_in_place = lambda: next(fresh)()

    out = {"shape": list(shape), "count": count}
    for name, fn in (("ms_loop_of_single_calls", loop), ("ms_one_batch_call", batch),
                     ("ms_one_prepared_batch_call", prepared), ("ms_one_prepared_batch_call_in_place", prepared_in_place)):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        out[name] = (time.perf_counter() - t0) * 1e3 / steps
    # what the GPU spends on one batch call, from the library's own events
    tr = mp.KernelTrace(8)
    with tr:
        batch()
    d = tr.durations_ms()
    tr.close()
    labels = {1: ["tiny_batch (one kernel for all)"], 3: ["colagg", "reduce", "colmap+search"],
              5: ["colagg", "reduce", "seeding+search", "l11_sweeps", "colmap"]}.get(
                  len(d), ["interval_%d" % k for k in range(len(d))])
    out["batch_kernel_ms_event_intervals"] = dict(zip(labels, d))
    return out


def host_description():
    """Logical CPUs this process may use, and the CPU model string of the host."""
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for ln in f:
                if ln.lower().startswith("model name"):
                    model = ln.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return usable, os.cpu_count() or usable, model


# ---- the all-cores leg of the CPU baseline: the paper's own decomposition (Sec. 6.2: a pool of
# workers over blocks of columns for the aggregate and for the per-column map, the vector
# projection in between on the main thread).  Worker processes are forked BEFORE this process
# touches the GPU and run nothing but the oracle's functions on their block of columns.
_POOL_Y = None      # the workload matrix, inherited by the forked workers
_POOL_X = None      # shared output buffer (multiprocessing.RawArray), inherited too


def _pool_aggregate(block):
    from oracle import mlproj_oracle as orc
    a, b = block
    return a, orc.column_norms(_POOL_Y[:, a:b], "inf")


def _pool_map(task):
    import numpy as np
    from oracle import mlproj_oracle as orc
    a, b, u = task
    n, m = _POOL_Y.shape
    X = np.frombuffer(_POOL_X, dtype=np.float32).reshape(n, m)
    for j in range(a, b):                      # x_j = P^inf_{u_j}(y_j), column by column
        X[:, j] = orc.project_linf_ball(_POOL_Y[:, j], u[j - a])
    return a


def cpu_all_cores(Y_host, eta, budget_s=12.0):
    """The oracle's three steps with the columns split over a pool of worker processes, one per
    usable core (the thread-pool decomposition of Sec. 6.2); the vector projection stays serial.
    Must run before the GPU is initialised (it forks).  Returns the timing record and X."""
    import multiprocessing as mp_
    import numpy as np
    from oracle import mlproj_oracle as orc
    global _POOL_Y, _POOL_X
    usable, _, _ = host_description()
    cap = os.environ.get("OMP_NUM_THREADS")
    workers = max(1, min(usable, int(cap)) if cap and cap.isdigit() else usable)
    n, m = Y_host.shape
    _POOL_Y = Y_host
    _POOL_X = mp_.RawArray("f", n * m)
    edges = [round(k * m / (4 * workers)) for k in range(4 * workers + 1)]   # four blocks per worker
    blocks = [(a, b) for a, b in zip(edges[:-1], edges[1:]) if b > a]
    times = []
    with mp_.get_context("fork").Pool(workers) as pool:
        t_all = time.perf_counter()
        while len(times) < 5 and (time.perf_counter() - t_all) < budget_s:
            t0 = time.perf_counter()
            v = np.empty(m, dtype=np.float32)
            for a, part in pool.imap_unordered(_pool_aggregate, blocks):       # step 1, parallel
                v[a:a + part.size] = part
            u64, tau = orc.project_l1_ball_nonneg(v, eta)                      # step 2, serial
            u = u64.astype(np.float32)
            for _ in pool.imap_unordered(_pool_map, [(a, b, u[a:b]) for a, b in blocks]):   # step 3, parallel
                pass
            times.append(time.perf_counter() - t0)
    X = np.frombuffer(_POOL_X, dtype=np.float32).reshape(n, m).copy()
    _POOL_Y = _POOL_X = None
    t = statistics.median(times)
    return {"cores_all": workers, "ms_all_cores": t * 1e3, "value_all_cores": 8.0 * n * m / t / 1e9,
            "runs_all_cores": len(times), "tau_all_cores": tau}, X


def cpu_baseline(Y_host, eta, x_timed, tau_gpu, budget_s=15.0):
    """The oracle as it stands, single numpy thread, on the headline workload with the radius
    the GPU runs used; its result also checks the X the last timed GPU step produced."""
    import numpy as np
    from oracle import mlproj_oracle as orc
    tensor = Y_host.ndim == 3
    run = orc.trilevel_l1infinf if tensor else orc.bilevel_l1inf
    times = []
    t_all = time.perf_counter()
    while len(times) < 5 and (time.perf_counter() - t_all) < budget_s:
        t0 = time.perf_counter()
        ref = run(Y_host, eta)
        times.append(time.perf_counter() - t0)
    t = statistics.median(times)
    err = np.abs(x_timed.astype(np.float64) - ref["X"])
    bar = 1e-5 * np.abs(ref["X"]) + 1e-6
    group_max = np.abs(x_timed).reshape(x_timed.shape[0], -1).max(axis=1) if tensor else np.abs(x_timed).max(axis=0)
    parity = {"max_abs_err": float(err.max()), "within_rtol1e-5_atol1e-6": bool((err <= bar).all()),
              "support_identical": bool(np.array_equal(group_max > 0, np.asarray(ref["u"]) > 0)),
              "tau_rel_err": abs(tau_gpu - ref["tau"]) / ref["tau"] if ref["tau"] > 0 else 0.0}
    usable, logical, model = host_description()
    return {"value": 8.0 * Y_host.size / t / 1e9, "unit": "GB/s", "ms": t * 1e3, "cores": 1, "kind": "oracle",
            "sample": "full %s workload, median of %d runs of oracle.%s" % ("x".join(map(str, Y_host.shape)), len(times), run.__name__),
            "nproc": usable, "logical_cpus": logical, "cpu_model": model,
            "gpu_x_vs_oracle": parity}, ref["X"]


def compact(x):
    """Floats to six significant digits, recursively (the last line stays under 2 KB)."""
    if isinstance(x, float):
        return float("%.6g" % x)
    if isinstance(x, dict):
        return {k: compact(v) for k, v in x.items()}
    if isinstance(x, (list, tuple)):
        return [compact(v) for v in x]
    return x


def summary_of(rec):
    """ms and fraction of the HBM peak (8 B/element model) of one detailed record."""
    out = {"ms": round(rec["ms"], 5)}
    if "frac_of_peak_rw" in rec:
        out["frac"] = round(rec["frac_of_peak_rw"], 4)
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    from paper_2405_02086_amd import workloads

    w, Y = workloads.make(args.workload)
    if args.variant != "l1inf":
        args.quick = True
    want_cpu = not (args.quick or args.no_cpu)
    tensor = len(w.shape) == 3
    all_cores = x_all = None
    if want_cpu and not tensor:
        # first, while this process has not touched the GPU: the leg that forks worker processes
        from oracle import mlproj_oracle as orc
        eta_cpu = float(np.float32(w.eta_frac * orc.norm_l1q(Y, "inf")))
        all_cores, x_all = cpu_all_cores(Y, eta_cpu)
        all_cores["eta_all_cores"] = eta_cpu

    import torch
    from paper_2405_02086_amd import binding as mp
    mp.lib()   # fail loudly if the HIP library is missing

    if tensor:
        head = bench_trilevel_head(torch, mp, Y, w.eta_frac, args.steps, args.warmup, keep_output=want_cpu)
    else:
        head = bench_bilevel(torch, mp, Y, args.variant, w.eta_frac, args.steps, args.warmup, keep_output=want_cpu)
    x_timed = head.pop("_x_timed", None)
    elems = Y.size
    what = "tri-level l1,inf,inf" if tensor else "bi-level " + {"l1inf": "l1,inf", "l12": "l1,2", "l11": "l1,1"}[args.variant]
    # the dominant kernel: the one that reads Y and writes X (8 B/element)
    kms = head["kernel_ms"]
    dom = max(kms, key=kms.get)
    dom_ms = kms[dom]
    if args.variant == "l11" and head.get("inner_sweeps") == 0 and dom == "colmap":
        # no lock-step sweep ran: the last kernel is the one that holds the columns in registers
        # (inner searches and soft-threshold), not the plain map pass
        dom = "l11_held (inner searches + map from registers)"
    traffic_ok = (args.workload in TRAFFIC_KIB and args.variant == "l1inf"
                  and mp.lib().mlproj_version() in TRAFFIC_VERSIONS)
    roofline = {
        "bound": "hbm", "kernel": "%s (%s; 8 B/element: reads Y, writes X)" % (dom, what),
        "achieved": 8.0 * elems / dom_ms / 1e6, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": 8.0 * elems / dom_ms / 1e6 / HBM_PEAK_GBS,
        "traffic": TRAFFIC_KIB[args.workload] * 1024.0 if traffic_ok else None,
        "traffic_source": "profiles/ (rocprofv3 --pmc, taken with library version %d)" % TRAFFIC_VERSIONS[0] if traffic_ok else None,
        "algorithmic_bytes": 8.0 * elems,
        "kernel_ms": dom_ms,
        "all_kernels_ms": {k: round(v, 5) for k, v in kms.items()},
    }
    line = {
        "metric": "effective HBM GB/s of one %s projection (8 B/element), cold caches" % what,
        "value": head["eff_GBps_rw"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: %s fp32 %s, entries %s, eta=%.2f*norm; cold (%d rotating buffer pairs)"
                               % (args.workload, "x".join(map(str, Y.shape)), "C-order" if tensor else "row-major",
                                  DIST_TEXT[w.dist], w.eta_frac, head["buffer_pairs"]),
                   "input_crc32": "%08x" % zlib.crc32(Y.tobytes())},
        "frac_of_hbm_peak": head["frac_of_peak_rw"], "ms_per_step_warm": head["ms_warm"],
        "roofline": roofline,
    }
    detail = {"headline": head,
              "generator": "numpy Generator(PCG64(%d)), see paper_2405_02086_amd/workloads.py" % w.seed}
    if not args.quick and not tensor:
        also = {}
        wb, Yb = workloads.make("square_16384")
        for variant, steps in (("l1inf", 20), ("l12", 20), ("l11", 5)):
            also["square_16384/" + variant] = bench_bilevel(torch, mp, Yb, variant, wb.eta_frac, steps, 3)
        # the same matrix kept in 16 bits (4 bytes per element in the effective figures, not 8)
        also["square_16384/l1inf/bf16"] = bench_bilevel(torch, mp, Yb, "l1inf", wb.eta_frac, 20, 3, storage="bf16")
        also["square_16384/l11/bf16"] = bench_bilevel(torch, mp, Yb, "l11", wb.eta_frac, 5, 3, storage="bf16")
        also["square_4096/l1inf/bf16"] = bench_bilevel(torch, mp, Y, "l1inf", w.eta_frac, 100, 10, storage="bf16")
        also["square_4096/l12"] = bench_bilevel(torch, mp, Y, "l12", w.eta_frac, 100, 10)
        also["square_4096/l11"] = bench_bilevel(torch, mp, Y, "l11", w.eta_frac, 50, 5)
        # the l2 and l_inf balls as outer norm (no iteration in the search)
        also["square_4096/l1inf/outer_l2"] = bench_bilevel(torch, mp, Y, "l1inf", w.eta_frac, 100, 10, outer=2)
        also["square_4096/l1inf/outer_linf"] = bench_bilevel(torch, mp, Y, "l1inf", w.eta_frac, 100, 10, outer="inf")
        # the weighted l1 ball as outer norm (its own one-workgroup search kernel, nothing fused)
        also["square_4096/l1inf/weighted"] = bench_bilevel(torch, mp, Y, "l1inf", w.eta_frac, 100, 10, weighted=True)
        also["square_4096/l11/weighted"] = bench_bilevel(torch, mp, Y, "l11", w.eta_frac, 50, 5, weighted=True)
        del Yb
        # the shape and distribution of the paper's own timing runs (Sec. 6.1): time against the radius
        wp, Yp = workloads.make("paper_1000x10000")
        for eta_abs in (0.25, 1.0, 4.0):
            also["paper_1000x10000/l1inf/eta=%g" % eta_abs] = bench_bilevel(torch, mp, Yp, "l1inf", None, 100, 10,
                                                                         eta_abs=eta_abs)
        # ... and the other two bi-level variants the paper times on it, at the middle radius
        for variant in ("l11", "l12"):
            also["paper_1000x10000/%s/eta=1" % variant] = bench_bilevel(torch, mp, Yp, variant, None, 100, 10,
                                                                       eta_abs=1.0)
        del Yp
        wt, Yt = workloads.make("tensor_256x256x256")
        for k, v in bench_tensor(torch, mp, Yt, wt.eta_frac, 100, 10).items():
            also["tensor_256x256x256/" + k] = v
        for name in ("tall_262144x256", "wide_256x262144"):
            wk, Yk = workloads.make(name)
            also[name + "/l1inf"] = bench_bilevel(torch, mp, Yk, "l1inf", wk.eta_frac, 50, 5)
            del Yk
        ws_, Ys_ = workloads.make("small_256x128")
        also["small_256x128/l1inf"] = bench_small(torch, mp, Ys_, ws_.eta_frac, 200, 20)
        also["batch/16x(256x128)"] = bench_batch(torch, mp, (256, 128), 16, 0.1, 100, 10)
        also["batch/16x(1024x1024)"] = bench_batch(torch, mp, (1024, 1024), 16, 0.1, 100, 10)
        also["batch/6x(4096x4096)"] = bench_batch(torch, mp, (4096, 4096), 6, 0.3, 30, 3)
        also["batch/16x(256x128)/l11"] = bench_batch(torch, mp, (256, 128), 16, 0.1, 100, 10, "l11")
        also["batch/16x(1024x1024)/l11"] = bench_batch(torch, mp, (1024, 1024), 16, 0.1, 100, 10, "l11")
        also["paper_size_sweep"] = bench_size_sweep(torch, mp, workloads, 50, 5)
        detail["also"] = also
        # the other workloads of the parity suite in the last line: ms per projection and the
        # fraction of the 8 TB/s peak on the 8 B/element model
        line["other_workloads"] = {
            "square_16384_l1inf": summary_of(also["square_16384/l1inf"]),
            "square_16384_l12": summary_of(also["square_16384/l12"]),
            "square_16384_l11": summary_of(also["square_16384/l11"]),
            "square_4096_l11": summary_of(also["square_4096/l11"]),
            "tall_262144x256": summary_of(also["tall_262144x256/l1inf"]),
            "wide_256x262144": summary_of(also["wide_256x262144/l1inf"]),
            "tensor_256x256x256": summary_of(also["tensor_256x256x256/trilevel_proj_l1infinf"]),
            "small_256x128": {"ms": round(also["small_256x128/l1inf"]["ms_eager"], 5)},
        }
    if want_cpu:
        base, x_ref = cpu_baseline(Y, head["eta"], x_timed, head["tau"])
        if all_cores is not None:
            base.update(all_cores)
            if all_cores["eta_all_cores"] == head["eta"]:
                base["all_cores_output_equals_one_thread_output"] = bool(np.array_equal(x_all, x_ref))
        line["cpu_baseline"] = base
    # Everything bulky first (its own stdout line, and a file where a results folder exists); the
    # LAST line is the compact record.
    blob = json.dumps({"detail": detail})
    print(blob)
    try:
        out_dir = os.path.join(ROOT, "gpurun_out")
        os.makedirs(out_dir, exist_ok=True)
        with open(os.path.join(out_dir, "bench_detail.json"), "w") as f:
            f.write(blob + "\n")
    except OSError:
        pass
    sys.stdout.flush()
    print(json.dumps(compact(line), separators=(",", ":")))


if __name__ == "__main__":
    main()
