#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: forward + gather-form backward of an element-wise
defined tensor, reported as tensor elements per second and as a fraction of the HBM roofline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3] [--no-others] [--no-cpu]

One "step" is one pass of the whole path (tad_eval_forward + tad_eval_backward, every gradient)
over one batch of seeded synthetic inputs that already live in HBM.  Prints ONE JSON line.
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

GRAPH_WORKLOADS = ("cfg1", "cfg5")   # steps of a few short launches: also timed as replays of a captured graph
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
FP32_VALU_TFLOPS = 157.3       # published vector fp32 peak (packed); 256 CUs x 2.4 GHz x 256 flop/clk
FP32_MFMA_TFLOPS = 157.3
PROFILE_EVERY = 25              # at most every 25th launch of the dominant kernel carries timing events (a timed launch delays
                                # its successor: every 7th cost the 25 us workload 3 us per step, every 25th nothing measurable);
                                # short runs time every (steps // 4)-th launch instead, so that several launches are averaged
ROTATE_BYTES = 640 << 20      # cycle over buffer sets beyond this footprint (> 2x the 256 MB last-level cache)
WARM_PASSES = 3                 # every buffer set is run this often before anything is timed, whatever --warmup says
MIN_WINDOW_MS = 20.0            # the workloads beside the headline are timed for at least this long (own step count)


# HBM traffic of the dominant kernel per launch, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs scaled by a plain
# 256 MiB copy in the same run (summaries under profiles/).  Each entry carries the SHA-256 prefix of the kernel source
# the counters were taken with; once that file changes the entry is stale and the bench line reports traffic = null.
MEASURED_TRAFFIC = {
    "cfg3": dict(source="kernels_worked.hip", sha256="c4542a3a73030316", fetch_bytes=521.5 * 2**20, write_bytes=9.5 * 2**20,
            summary="profiles/worked_8192x8192x5_f32.md"),
    "cfg4": dict(source="kernels_mfma.hip", sha256="a837d56d973eb5ad", fetch_bytes=160.5 * 2**20, write_bytes=32.2 * 2**20,
            summary="profiles/worked_mfma_4096x4096x256_f32.md"),
    "matmul": dict(source="kernels_contract.hip", sha256="44643592ea5bb39b", fetch_bytes=626.4 * 2**20, write_bytes=64.0 * 2**20,
            summary="profiles/contraction_4096x4096x4096_f32.md"),
    "cfg2_1": dict(source="kernels_patterns.hip", sha256="82a47a45178e317d", fetch_bytes=64.3 * 2**20, write_bytes=0.1 * 2**20,
            summary="profiles/row_reduce_4096x4096_f32.md"),
    "cfg2_2": dict(source="kernels_patterns.hip", sha256="82a47a45178e317d", fetch_bytes=1.1 * 2**20, write_bytes=256.2 * 2**20,
            summary="profiles/diagonal_8192_f32.md"),
    "cfg2_3": dict(source="kernels_patterns.hip", sha256="82a47a45178e317d", fetch_bytes=64.1 * 2**20, write_bytes=0.5 * 2**20,
            summary="profiles/antidiagonal_4096x4096_f32.md"),
    "cfg5": dict(source="kernels_strided.hip", sha256="748ea7db15a78ccd", fetch_bytes=20.6 * 2**20, write_bytes=8.5 * 2**20,
            summary="profiles/strided_32x128x128_f32.md"),
}


def workload(name):
    from paper_1711_01348_amd import workloads as wl
    table = {
        "cfg1": wl.config1, "cfg2_1": lambda: wl.config2(1), "cfg2_2": lambda: wl.config2(2),
        "cfg2_3": lambda: wl.config2(3), "cfg3": wl.config3, "cfg4": wl.config4, "cfg5": wl.config5,
        "matmul": wl.matmul_workload,
    }
    return table[name]()


def accounting(name, w):
    """Compulsory work of one forward+backward step.

    Returns (tensor elements, bytes, dominant) where dominant describes the kernel the roofline entry is
    computed for: name, bound ("hbm" or "mfma"), algorithmic bytes or flops per launch, launches per step.
    """
    import numpy as np
    e = w.expr
    nf = int(np.prod(e.f_shape))
    small = sum(int(np.prod(a.shape)) for a in e.args)
    es = 4 if e.dtype == "f32" else 8
    if name in ("cfg3", "cfg4", "cfg1"):
        I, J = e.f_shape
        K = e.sums[0][1] + 1
        cdense = int(np.prod(e.args[2].shape))
        small_rw = 2 * (small - cdense) + I          # a, b, d read; da, db, dd written; diagonal of c read
        elems = nf + nf + nf + cdense + small_rw      # write f; read df; read f; write dense dc
        if name == "cfg4":
            # expanded form on the matrix cores: a.b^T, G b and (cG)^T a, 2 I J K flops each
            dom = dict(kernel="k_mfma_backward", bound="mfma", per_launch=2.0 * I * J * K, launches=2,
                       step_flops=6.0 * I * J * K)
        elif name == "cfg3":
            dom = dict(kernel="k_worked_backward", bound="hbm", per_launch=2 * nf * es, launches=1)
        else:
            dom = dict(kernel="k_generic_gather_listed", bound="hbm", per_launch=0, launches=1)   # four gradients, one launch
    elif name == "cfg2_1":
        elems = nf + nf + 2 * small                   # write f; read df; x read, dx written
        dom = dict(kernel="k_rowreduce_backward", bound="hbm", per_launch=nf * es, launches=1)
    elif name == "cfg2_2":
        elems = small + 3 * nf                        # write dense dx; diagonal read, f written, df read
        dom = dict(kernel="k_diagonal_backward", bound="hbm", per_launch=small * es, launches=1)
    elif name == "cfg2_3":
        elems = nf + nf + 2 * small
        dom = dict(kernel="k_antidiag_backward", bound="hbm", per_launch=nf * es, launches=1)
    elif name == "matmul":
        I, J = e.f_shape
        K = e.sums[0][1] + 1
        elems = 2 * small + nf + nf + small           # fwd: read x, y, write f; bwd: read df, x, y, write dx, dy
        dom = dict(kernel="k_contract", bound="mfma", per_launch=2.0 * I * J * K, launches=3,
                   step_flops=6.0 * I * J * K)
    elif name == "cfg5":
        nx = int(np.prod(e.args[0].shape))
        elems = nx + nf + 2 * nf + nx + nx + 18       # fwd: read x, write f; bwd: read df, f; write dx; read x (dw)
        dom = dict(kernel="k_strided_backward", bound="hbm", per_launch=(2 * nf + 2 * nx) * es, launches=1)
    else:
        raise ValueError(name)
    return elems, elems * es, dom


def run_gpu(name, steps, warmup, rotate_bytes=0, min_window_ms=0.0, grads=None):
    """Time `steps` forward+backward passes.  With rotate_bytes > 0 the step cycles over enough independent
    buffer sets to exceed that footprint, so that a workload smaller than the last-level cache still streams
    from HBM.  With min_window_ms > 0 the step count is raised until the timed region lasts that long (a 1.5 ms
    window of 20 short steps measures the start of the run, not the steady state)."""
    import ctypes
    import torch
    from paper_1711_01348_amd import binding as B
    w = workload(name)
    plan = B.Plan(w.expr)
    dev = torch.device("cuda:0")
    elems, nbytes, dom = accounting(name, w)
    # every workload starts from fresh allocations, as if it were run alone: buffers carved out of the blocks that a
    # previous, larger workload left in the caching allocator measured up to 20 % slower for the smallest workloads
    torch.cuda.empty_cache()

    def make_set():
        args = [torch.from_numpy(a).to(dev) for a in w.arg_list()]
        df = torch.from_numpy(w.df).to(dev)
        f = torch.empty(tuple(w.expr.f_shape), dtype=df.dtype, device=dev)
        out = [torch.empty_like(a) if (grads is None or p in grads) else None for p, a in enumerate(args)]
        return args, df, f, out, plan.workspace(dev)

    sets = [make_set()]
    foot = sum(t.numel() * t.element_size() for t in sets[0][0] + [sets[0][1], sets[0][2]] + [o for o in sets[0][3] if o is not None])
    while rotate_bytes and foot * len(sets) < rotate_bytes and len(sets) < 64:
        sets.append(make_set())

    def step(i):
        args, df, f, out, ws = sets[i % len(sets)]
        plan.forward(args, out=f, ws=ws)
        plan.backward(args, f, df, wanted=[o is not None for o in out], out=out, ws=ws)

    warm = max(warmup, WARM_PASSES * len(sets))      # first touches of a buffer set are never part of the timed region
    for i in range(warm):
        step(i)
    torch.cuda.synchronize()
    if min_window_ms:
        pilot = max(steps, len(sets))
        t0 = time.perf_counter()
        for i in range(pilot):
            step(i)
        torch.cuda.synchronize()
        per_step_ms = (time.perf_counter() - t0) * 1e3 / pilot
        steps = max(steps, int(min_window_ms / per_step_ms) + 1)
    every = max(1, min(PROFILE_EVERY, steps // 4))
    families = {"forward": plan.forward_family, "backward": [plan.query(p)["family"] for p in range(len(w.expr.args))]}
    if dom["per_launch"]:   # a workload without a roofline figure (cfg1: all latency) runs without timed launches
        B._check(B.lib.tad_profile_begin(dom["kernel"].encode(), every), "tad_profile_begin")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms, n = ctypes.c_double(0), ctypes.c_int(0)
    B._check(B.lib.tad_profile_end(ctypes.byref(ms), ctypes.byref(n)), "tad_profile_end")
    dom_ms = ms.value / n.value if n.value else None
    # forward / backward split (outside the timed region) with events on the stream the kernels run on
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    args, df, f, out, ws = sets[0]
    ev[0].record()
    plan.forward(args, out=f, ws=ws)
    ev[1].record()
    plan.backward(args, f, df, wanted=[o is not None for o in out], out=out, ws=ws)
    ev[2].record()
    torch.cuda.synchronize()
    ms_step = (t1 - t0) * 1e3 / steps
    extra = {}
    if name in GRAPH_WORKLOADS:
        # launch-bound workloads: the same steps captured once per buffer set into a HIP graph and replayed (both
        # evaluation calls only enqueue kernels), which is how a caller with steps this short would issue them
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graphs = []
        for i in range(len(sets)):
            with torch.cuda.stream(side):
                step(i)
            side.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                step(i)
            graphs.append(g)
        for k in range(WARM_PASSES * len(graphs)):
            graphs[k % len(graphs)].replay()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for k in range(steps):
            graphs[k % len(graphs)].replay()
        torch.cuda.synchronize()
        extra["ms_per_step_graph_replay"] = (time.perf_counter() - t2) * 1e3 / steps
        del graphs
    if name == "cfg4":
        # the same forward pass in the direct form on the vector ALUs, for comparison with the expanded form on MFMA
        pd = B.Plan(w.expr, direct_form=True)
        for _ in range(3):
            pd.forward(args, out=f, ws=ws)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            pd.forward(args, out=f, ws=ws)
        e1.record()
        torch.cuda.synchronize()
        extra["ms_forward_direct_valu_form"] = e0.elapsed_time(e1) / 10
    return dict(name=name, workload=w.name, ms_per_step=ms_step, elements=elems, bytes=nbytes,
                elements_per_s=elems / (ms_step * 1e-3), algorithmic_gbs=nbytes / (ms_step * 1e-3) / 1e9,
                ms_forward=ev[0].elapsed_time(ev[1]), ms_backward=ev[1].elapsed_time(ev[2]),
                dominant=dom, dominant_ms=dom_ms, dominant_launches=n.value, timed_every=every, steps=steps,
                warm_steps=warm, families=families,
                dtype=w.expr.dtype, buffer_sets=len(sets), footprint_bytes_per_set=foot, extra=extra)


def measured_traffic(name):
    """Per-launch HBM bytes of the dominant kernel from the committed counter runs, or None if the kernel source
    has changed since."""
    import hashlib
    t = MEASURED_TRAFFIC.get(name)
    if not t:
        return None
    src = os.path.join(ROOT, "paper_1711_01348_amd", "csrc", t["source"])
    try:
        with open(src, "rb") as fh:
            if hashlib.sha256(fh.read()).hexdigest()[:16] != t["sha256"]:
                return None
    except OSError:
        return None
    return t["fetch_bytes"] + t["write_bytes"]


def roofline(r):
    dom, ms = r["dominant"], r["dominant_ms"]
    if not ms or not dom["per_launch"]:
        return {"bound": dom["bound"], "kernel": dom["kernel"], "achieved": None, "peak": None, "unit": None,
                "frac": None, "traffic": None}
    if dom["bound"] == "mfma":
        achieved, peak, unit = dom["per_launch"] / (ms * 1e-3) / 1e12, FP32_MFMA_TFLOPS, "TFLOP/s"
    else:
        achieved, peak, unit = dom["per_launch"] / (ms * 1e-3) / 1e9, HBM_PEAK_GBS, "GB/s"
    return {"bound": dom["bound"], "kernel": dom["kernel"], "achieved": achieved, "peak": peak, "unit": unit,
            "frac": achieved / peak, "traffic": measured_traffic(r["name"]), "avg_kernel_ms": ms, "launches": r["dominant_launches"], "timed_every": r["timed_every"],
            "algorithmic_per_launch": dom["per_launch"]}


def run_cpu_oracle(name):
    """The fp64 oracle as it stands, on the host cores, on the same workload: the whole workload with the function
    indices split over the cores (cfg3 takes a few seconds), and one thread on a contiguous block of rows of it."""
    import ctypes
    import oracle
    w = workload(name)
    nproc = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    nthreads = min(oracle.max_threads(), 16, nproc)      # the share of the host that belongs to one GPU
    t0 = time.perf_counter()
    oracle.forward(w.expr, w.arg_list())
    oracle.backward(w.expr, w.arg_list(), w.df, nthreads=nthreads)
    t = time.perf_counter() - t0
    elems, _, _ = accounting(name, w)
    out = dict(value=elems / t, unit="elements/s", cores=nthreads, nproc=nproc, kind="oracle",
               sample=f"whole workload {w.name}: forward + brute-force scatter backward, fp64, {t:.1f} s on {nthreads} threads")
    if name in ("cfg3", "cfg4") and w.expr.f_shape[0] >= 1024:
        # one thread: rows 0 .. n-1 of the same tensors (an n x J x K worked expression: a, c, d and df cut to those rows)
        from paper_1711_01348_amd import workloads as wl
        I, J = w.expr.f_shape
        K = w.expr.sums[0][1] + 1
        n = I // 16 if name == "cfg3" else I // 128
        a_, b_, c_, d_ = w.arg_list()
        sub = wl.worked_expr(n, J, K, w.expr.dtype)
        xs = [a_[:n], b_, c_[:n, :n].copy(), d_[:n + K - 1]]
        try:
            omp = ctypes.CDLL("libgomp.so.1")
        except OSError:
            return out
        before = oracle.max_threads()
        omp.omp_set_num_threads(1)               # the forward pass takes its thread count from the OpenMP runtime
        t0 = time.perf_counter()
        oracle.forward(sub, xs)
        oracle.backward(sub, xs, w.df[:n], nthreads=1)
        t1 = time.perf_counter() - t0
        omp.omp_set_num_threads(before)
        out["single_thread_value"] = elems * (n / I) / t1
        out["single_thread_sample"] = f"rows 0..{n - 1} of {I} of the same workload, one thread, {t1:.1f} s"
    return out


def vendor_product(torch):
    """torch.mm in fp32 on random normal operands, HIP events around 50 calls after 10 warm-up calls."""
    torch.backends.cuda.matmul.allow_tf32 = False
    for m, n, k in ((4096, 4096, 4096), (4096, 4096, 256), (4096, 256, 4096)):
        x = torch.randn(m, k, device="cuda:0")
        y = torch.randn(k, n, device="cuda:0")
        out = torch.empty(m, n, device="cuda:0")
        for _ in range(10):
            torch.mm(x, y, out=out)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(50):
            torch.mm(x, y, out=out)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / 50 * 1e3
        print(json.dumps({"vendor_product": "torch.mm fp32", "shape_mnk": [m, n, k], "us": us,
                          "tflops": 2.0 * m * n * k / us / 1e6, "frac_of_mfma_peak": 2.0 * m * n * k / us / 1e6 / FP32_MFMA_TFLOPS}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--no-others", action="store_true", help="skip the other configurations (extra keys)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--grads", default=None,
                    help="operand numbers whose gradients the backward call computes (e.g. 0 or 0,2); default: all. "
                         "For looking at one gradient's kernels alone; the accounting of elements stays that of the whole step")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy 5 times (reference point for HBM byte counters)")
    ap.add_argument("--vendor-product", action="store_true",
                    help="instead of a workload, time torch.mm (the vendor's fp32 product) at the shapes of the matmul "
                         "workload and of cfg4's three contractions: a yardstick for the matrix-core kernels, one line each")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this library runs on ONE GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)

    if a.vendor_product:
        vendor_product(torch)
        return
    if a.calibrate_copy:
        src = torch.empty(64 << 20, dtype=torch.float32, device="cuda:0").normal_()
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    rot = 0 if a.workload == "cfg3" else ROTATE_BYTES
    only = None if a.grads is None else [int(t) for t in a.grads.split(",")]
    r = run_gpu(a.workload, a.steps, a.warmup, rotate_bytes=rot, grads=only)
    out = {
        "metric": "fwd+bwd tensor elements/s; achieved HBM GB/s or FLOP/s vs MI355X peak",
        "value": r["elements_per_s"], "unit": "elements/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": r["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": r["dtype"], "data": "synthetic",
        "config": {"workload": r["workload"], "families": r["families"],
                   "elements_per_step": r["elements"], "algorithmic_bytes_per_step": r["bytes"],
                   "ms_forward": r["ms_forward"], "ms_backward": r["ms_backward"],
                   "step_algorithmic_GBs": r["algorithmic_gbs"],
                   "step_frac_of_hbm_peak": r["algorithmic_gbs"] / HBM_PEAK_GBS,
                   "buffer_sets": r["buffer_sets"], "gradients": "all" if only is None else only},
        "roofline": roofline(r),
    }
    out["config"].update(r["extra"])
    if not a.no_others:
        per = {}
        for name in ("cfg1", "cfg2_1", "cfg2_2", "cfg2_3", "cfg4", "cfg5", "matmul"):
            if name == a.workload:
                continue
            try:
                q = run_gpu(name, a.steps, a.warmup, rotate_bytes=ROTATE_BYTES, min_window_ms=MIN_WINDOW_MS)
                e = {k: q[k] for k in ("workload", "steps", "warm_steps", "ms_per_step", "ms_forward", "ms_backward", "elements_per_s",
                                       "algorithmic_gbs", "families", "buffer_sets")}
                e["frac_of_hbm_peak"] = q["algorithmic_gbs"] / HBM_PEAK_GBS
                if q["dominant"]["bound"] == "mfma":
                    tf = q["dominant"]["step_flops"] / (q["ms_per_step"] * 1e-3) / 1e12
                    e["step_TFLOPs"] = tf
                    e["step_frac_of_fp32_mfma_peak"] = tf / FP32_MFMA_TFLOPS
                e.update(q["extra"])
                e["roofline"] = roofline(q)
                per[name] = e
            except Exception as ex:  # report, never hide
                per[name] = {"error": repr(ex)}
        out["per_config"] = per
    if not a.no_cpu:
        out["cpu_baseline"] = run_cpu_oracle(a.workload)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
