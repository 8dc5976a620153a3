#!/usr/bin/env python3
"""bench.py -- throughput of the AdaComp pack/unpack hot path on one MI355X.

One "step" is one mini-batch of the whole hot path on one GPU: every simulated learner runs
adacomp_compress on its own gradient and residue (Algorithm 2 of the AdaComp paper), then one
adacomp_unpack_accumulate sums all learners' packets into a dense gradient (unpack() of
Algorithm 1).  Inputs are seeded synthetic gradients already resident in HBM when the clock starts.

Every learner reads a gradient it has not seen before at every timed step (n_learners + steps - 1
buffers, learner k reads buffer k + t at step t), all generated and uploaded before the clock starts.

Prints ONE JSON line.  `value` = bytes of float32 gradient compressed and unpacked per second
(n_learners * 4 * n_elems per step).  `roofline` prices the dominant kernel (k_fused, the
streaming pass of compress) by its algorithmic bytes, 12 per element (read dW, read residue,
write residue), against the MI355X's 8 TB/s HBM peak, with its duration measured by HIP events
on the launch stream inside the timed region; beside the published peak the line carries what this
GPU sustains on a bare in-place triad (the best of 8, 6, 4 and 3 workgroups resident per compute
unit) and a bare fill with the same access pattern (`device_triad_GBs`, `device_fill_GBs`), measured
in the same run.  `cpu_baseline` times the CPU oracle, as it stands,
on a bounded sample of the same workload; `parity_checked` says whether step 0 of the calls that
were timed gave, bit for bit, the packets, residues and dense sum that oracle run produced (the
run exits non-zero if not); `per_config` holds the other four configurations, each as configured.
Beside these, never as `value`: `unpack_update` (the
fused unpack + average + optimizer step) and `lazy_residue` (the same steps through
adacomp_compress_batch_lazy, with the residue sync inside its timed region).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
MAX_GRAD_BUFFERS = 96  # gradient buffers held at most (48 GB on the largest workload)
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "k_fused_hbm_traffic.txt")


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def measured_traffic(workload_name):
    """HBM bytes per k_fused launch from the committed rocprofv3 --pmc summary, if there is one
    for this workload (lines 'workload: <name>' and 'traffic_bytes_per_launch: <int>')."""
    try:
        wl, val = None, None
        for line in open(TRAFFIC_FILE):
            if line.startswith("workload:"):
                wl = line.split(":", 1)[1].strip()
            if line.startswith("traffic_bytes_per_launch:") and wl == workload_name:
                val = int(float(line.split(":", 1)[1]))
        return val
    except OSError:
        return None


def small_config(wl, dev, threads, L, binding, A, W, torch, ctypes, repeats=5):
    """One of the smaller configurations exactly as configured: wl.n_learners learners, wl.n_steps
    steps from zero residues, a fresh gradient per learner and step (n + K - 1 buffers), one
    adacomp_compress_batch and one adacomp_unpack_accumulate per step.  The whole sequence is run
    `repeats` times from the same initial state (after one untimed run) and the median is reported."""
    n, K = wl.n_learners, wl.n_steps
    table, n_total, n_params = wl.table(), wl.n_total, wl.n_params
    grads = [torch.from_numpy(W.gradient(wl, i, 0, seed=0, threads=threads)).to(dev) for i in range(n + K - 1)]
    ws = torch.zeros(A.adacomp_workspace_bytes_batch(table, n), dtype=torch.uint8, device=dev)
    A.adacomp_workspace_init(table, ws)
    bound = A.adacomp_packet_bound(table)
    residue = [torch.zeros(n_total, dtype=torch.float32, device=dev) for _ in range(n)]
    packets = [torch.zeros(bound, dtype=torch.uint8, device=dev) for _ in range(n)]
    dense = torch.zeros(n_total, dtype=torch.float32, device=dev)
    vp = ctypes.c_void_p
    layers_c = binding.layer_array(table)
    stream = vp(torch.cuda.current_stream().cuda_stream)
    ws_p, ws_n = vp(ws.data_ptr()), ws.numel()
    pk_ptrs = (vp * n)(*[p.data_ptr() for p in packets])
    res_ptrs = (vp * n)(*[r.data_ptr() for r in residue])
    grad_ptrs = [(vp * n)(*[grads[k + t].data_ptr() for k in range(n)]) for t in range(K)]
    dense_p = vp(dense.data_ptr())
    times = []
    try:
        for rep in range(repeats + 1):
            for r in residue:
                r.zero_()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for t in range(K):
                rc = L.adacomp_compress_batch(layers_c, len(table), n, grad_ptrs[t], res_ptrs, pk_ptrs, bound, ws_p, ws_n, stream)
                if rc:
                    raise RuntimeError(f"adacomp_compress_batch: {rc}")
                rc = L.adacomp_unpack_accumulate(layers_c, len(table), pk_ptrs, n, dense_p, ws_p, ws_n, stream)
                if rc:
                    raise RuntimeError(f"adacomp_unpack_accumulate: {rc}")
            torch.cuda.synchronize()
            if rep:
                times.append((time.perf_counter() - t0) * 1e3 / K)
        times.sort()
        ms = times[len(times) // 2]
        n_sel = total_bytes = paper_bits = 0
        for p in packets:   # the last step's packets
            head, recs = A.read_packet_summary(p)
            n_sel += int(head["n_selected"])
            total_bytes += int(head["total_bytes"])
            paper_bits += int(sum(int(r["word_bits"]) * int(r["n_selected"]) for r in recs))
        pbar = total_bytes / n
        step_alg = n * (12 * n_params + pbar) + 4 * n_params + n * pbar
        return {"configuration": wl.index, "n_learners": n, "steps": K, "n_elems": n_params,
                "ms_per_step": round(ms, 4), "value": round(n * 4 * n_params / (ms * 1e-3) / 1e9, 2), "unit": "GB/s",
                "hbm_frac_step_algorithmic": round(step_alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                "compression_last_step": {"paper_accounting": round(32.0 * n_params * n / max(1, paper_bits), 2),
                                          "wire": round(4.0 * n_params * n / max(1, total_bytes), 2)},
                "timing": f"median of {repeats} runs of all {K} steps from zero residues, host clock around the run"}
    finally:
        A.adacomp_workspace_release(ws)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=5, help="1..5 (5 = speech-DNN FC stack, the metric's configuration)")
    ap.add_argument("--learners", type=int, default=0, help="override the workload's learner count")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true", help="do not bracket k_fused with HIP events")
    ap.add_argument("--no-lazy-leg", action="store_true", help="skip the extra leg through adacomp_compress_batch_lazy")
    ap.add_argument("--no-per-config", action="store_true", help="skip the per_config leg (configurations 1-4 as configured)")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of one step captured in a HIP graph (for the small, launch-bound workloads; "
                         "no roofline object, since events cannot be read back from a graph)")
    ap.add_argument("--batch", choices=["on", "off"], default="on",
                    help="on: one adacomp_compress_batch call per step (the library launches the streaming kernel "
                         "once per learner for large gradients and once per call for small ones; scan and placement "
                         "cover all learners); off: one adacomp_compress call per learner")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (simulated learners are separate buffers on "
                 "one device; there is no collective path) -- use --gpus 1")

    import numpy as np
    import torch

    import adacomp_workloads as W
    import paper_1712_02679_amd as A
    from paper_1712_02679_amd import binding

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; libadacomp has no CPU path")
    dev = "cuda:0"
    torch.cuda.set_device(0)
    wl = W.workload(args.workload)
    n_learners = args.learners or wl.n_learners
    table, n_total, n_params = wl.table(), wl.n_total, wl.n_params
    K, Wm = args.steps, args.warmup
    args.no_batch = args.batch == "off"
    threads = min(16, os.cpu_count() or 1)

    # ---- inputs: a fresh seeded draw for every (learner, step): n_learners + K - 1 gradient buffers,
    #      learner k reads buffer k + t at step t, so within the timed region no learner ever sees a
    #      gradient twice and no step uses a buffer twice.  All of it is generated and uploaded
    #      before the clock starts.  (Very long runs wrap around after MAX_GRAD_BUFFERS; the line says so.)
    t0 = time.time()
    n_buf = min(n_learners + max(K, Wm, 1) - 1, max(n_learners, MAX_GRAD_BUFFERS))
    grads = []
    for i in range(n_buf):
        g = W.gradient(wl, i, 0, seed=0, threads=threads)
        grads.append(torch.from_numpy(g).to(dev))
    fresh = n_buf >= n_learners + K - 1
    log(f"{wl.name}: {n_params} elements x {n_buf} gradient buffers ({n_learners} learners, {K} steps) generated and uploaded in {time.time() - t0:.1f}s")

    ws = torch.zeros(A.adacomp_workspace_bytes_batch(table, n_learners), dtype=torch.uint8, device=dev)
    A.adacomp_workspace_init(table, ws)
    bound = A.adacomp_packet_bound(table)
    residue = [torch.zeros(n_total, dtype=torch.float32, device=dev) for _ in range(n_learners)]
    packets = [torch.zeros(bound, dtype=torch.uint8, device=dev) for _ in range(n_learners)]
    dense = torch.zeros(n_total, dtype=torch.float32, device=dev)
    layers_c = binding.layer_array(table)

    L = binding.lib()
    import ctypes
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if args.graph:
        args.no_kernel_events = True
    ws_p, ws_n = ctypes.c_void_p(ws.data_ptr()), ws.numel()
    pk_ptrs = (ctypes.c_void_p * n_learners)(*[p.data_ptr() for p in packets])

    vp = ctypes.c_void_p
    res_ptrs = (vp * n_learners)(*[r.data_ptr() for r in residue])
    n_sets = n_buf - n_learners + 1   # gradient sets: set t holds the buffers of step t
    grad_ptrs = [(vp * n_learners)(*[grads[k + t].data_ptr() for k in range(n_learners)]) for t in range(n_sets)]

    cur = {"stream": stream}   # the stream the calls go to: torch's current one, or the capture stream

    def compress_all(t):
        stream = cur["stream"]
        if not args.no_batch:
            rc = L.adacomp_compress_batch(layers_c, len(table), n_learners, grad_ptrs[t % n_sets], res_ptrs,
                                          pk_ptrs, bound, ws_p, ws_n, stream)
            if rc:
                raise RuntimeError(f"adacomp_compress_batch: {rc}")
            return
        for k in range(n_learners):
            rc = L.adacomp_compress(layers_c, len(table), ctypes.c_void_p(grads[k + t % n_sets].data_ptr()),
                                    ctypes.c_void_p(residue[k].data_ptr()), ctypes.c_void_p(packets[k].data_ptr()),
                                    bound, ws_p, ws_n, stream)
            if rc:
                raise RuntimeError(f"adacomp_compress: {rc}")

    def unpack_all():
        rc = L.adacomp_unpack_accumulate(layers_c, len(table), pk_ptrs, n_learners,
                                         ctypes.c_void_p(dense.data_ptr()), ws_p, ws_n, cur["stream"])
        if rc:
            raise RuntimeError(f"adacomp_unpack_accumulate: {rc}")

    # ---- plain device copy of one gradient (8 B per element): the calibration kernel for the HBM
    #      byte counters, and the copy bandwidth this GPU reaches, for context ----------------------
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    A.adacomp_copy_f32(dense, grads[0], n_total)
    c0.record()
    for _ in range(5):
        A.adacomp_copy_f32(dense, grads[0], n_total)
    c1.record()
    torch.cuda.synchronize()
    copy_gbs = 8.0 * n_total * 5 / (c0.elapsed_time(c1) * 1e-3) / 1e9
    # the two streaming ceilings of this GPU with the access pattern of the hot kernels and nothing
    # else: an in-place x <- x + y (12 B per element, what k_fused moves) and a fill (4 B per element,
    # what the dense sum writes); `dense` is scratch here, unpack overwrites it
    n4 = n_total // 4 * 4
    # The triad is measured with 8, 6, 4 and 3 workgroups resident per compute unit (HBM serves it
    # better with fewer bytes in flight); the ceiling is the best of them.
    ceilings, triad_by_resident = {}, {}
    calls = [("triad_%d" % r, (lambda r=r: A.adacomp_triad_resident_f32(dense, grads[0], r, n4)), 12.0) for r in (8, 6, 4, 3)]
    calls.append(("fill", lambda: A.adacomp_fill_f32(dense, 0.0, n4), 4.0))
    for name, call, bytes_per_elem in calls:
        call()
        c0.record()
        for _ in range(5):
            call()
        c1.record()
        torch.cuda.synchronize()
        rate = bytes_per_elem * n4 * 5 / (c0.elapsed_time(c1) * 1e-3) / 1e9
        if name.startswith("triad_"):
            triad_by_resident[name[6:]] = round(rate, 1)
            ceilings["triad"] = max(ceilings.get("triad", 0.0), rate)
        else:
            ceilings[name] = rate

    # ---- warm-up on the same buffers, then residues back to zero (training start) ---------------
    for t in range(Wm):
        compress_all(t)
        unpack_all()
    torch.cuda.synchronize()
    for r in residue:
        r.zero_()
    torch.cuda.synchronize()

    # ---- optional: one step (gradient set 0) captured in a HIP graph, replayed K times ----------------
    graph = None
    if args.graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            cur["stream"] = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
            compress_all(0)
            unpack_all()
        cur["stream"] = stream
        torch.cuda.synchronize()

    # ---- timed region ------------------------------------------------------------------------------
    use_events = not args.no_kernel_events
    # every 11th k_fused launch (coprime with the learner counts in use, so it rotates through the
    # learners): an event pair around a launch costs the queue about 8 us, and at every 5th launch
    # that was 0.6 % of the step
    A.adacomp_timing_enable(11 if use_events else 0)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(K)]
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for t in range(K):
        if graph is not None:
            graph.replay()
            continue
        ev[t][0].record()
        compress_all(t)
        ev[t][1].record()
        unpack_all()
        ev[t][2].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    if graph is not None:   # no per-call split inside a graph: record once around nothing so the sums below read 0
        for t in range(K):
            for e in ev[t]:
                e.record()
        torch.cuda.synchronize()
    fused_ms, fused_n, fused_learners = A.adacomp_timing_read() if use_events else (0.0, 0, 0)
    A.adacomp_timing_enable(0)

    compress_ms = sum(ev[t][0].elapsed_time(ev[t][1]) for t in range(K)) / K
    unpack_ms = sum(ev[t][1].elapsed_time(ev[t][2]) for t in range(K)) / K
    if graph is not None:
        compress_ms = unpack_ms = float("nan")   # a replay is one submission: no split
    ms_per_step = elapsed * 1e3 / K
    log("per step compress ms: " + " ".join(f"{ev[t][0].elapsed_time(ev[t][1]):.3f}" for t in range(K)))
    log("per step unpack   ms: " + " ".join(f"{ev[t][1].elapsed_time(ev[t][2]):.3f}" for t in range(K)))
    grad_bytes_per_step = n_learners * 4 * n_params
    value = grad_bytes_per_step / (ms_per_step * 1e-3) / 1e9

    # ---- compression achieved at the last timed step (headers only: tiny copies) -------------------
    n_sel = total_bytes = 0
    paper_bits = 0
    for p in packets:
        head, recs = A.read_packet_summary(p)
        assert int(head["status"]) == 0
        n_sel += int(head["n_selected"])
        total_bytes += int(head["total_bytes"])
        paper_bits += int(sum(int(r["word_bits"]) * int(r["n_selected"]) for r in recs))
    packet_bytes_mean = total_bytes / n_learners
    ratio_paper = 32.0 * n_params * n_learners / max(1, paper_bits)
    ratio_wire = 4.0 * n_params * n_learners / max(1, total_bytes)

    # ---- roofline of the dominant kernel ------------------------------------------------------------
    per_launch = fused_learners // fused_n if fused_n else 1  # learners one k_fused launch covers
    alg_bytes_launch = 12 * n_params * per_launch  # k_fused: read dW, read residue, write residue, 4 B each
    roofline = None
    if use_events and fused_n:
        dur_ms = fused_ms / fused_n
        achieved = alg_bytes_launch / (dur_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "k_fused", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "traffic": (measured_traffic(wl.name) or 0) * per_launch or None,
                    "traffic_source": "committed rocprofv3 --pmc summary profiles/k_fused_hbm_traffic.txt (not a counter of this run)",
                    "algorithmic_bytes_per_launch": alg_bytes_launch, "learners_per_launch": per_launch,
                    "avg_launch_ms": round(dur_ms, 5), "launches": int(fused_n),
                    "frac_of_measured_triad": round(achieved / ceilings["triad"], 4)}
    # whole step by algorithmic bytes: n * (12 N + P) + 4 N + n * P
    step_alg_bytes = n_learners * (12 * n_params + packet_bytes_mean) + 4 * n_params + n_learners * packet_bytes_mean
    step_frac = step_alg_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS

    # ---- the follow-on row: unpack + average + optimizer step in one pass (not part of `value`) -------
    upd = {}
    try:
        wts = torch.zeros(n_total, dtype=torch.float32, device=dev)
        st1 = torch.zeros(n_total, dtype=torch.float32, device=dev)
        st2 = torch.zeros(n_total, dtype=torch.float32, device=dev)
        for name, kind, st2_arg, bytes_per_elem in (("sgd_momentum", binding.OPT_SGD_MOMENTUM, None, 16),
                                                    ("adam", binding.OPT_ADAM, st2, 24)):
            A.adacomp_unpack_update(table, packets, None, wts, st1, st2_arg, ws, kind, 1e-3, momentum=0.9,
                                    bias1=0.1, bias2=0.001)
            u0, u1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            u0.record()
            for _ in range(5):
                A.adacomp_unpack_update(table, packets, None, wts, st1, st2_arg, ws, kind, 1e-3, momentum=0.9,
                                        bias1=0.1, bias2=0.001)
            u1.record()
            torch.cuda.synchronize()
            ms = u0.elapsed_time(u1) / 5
            upd[name] = {"ms": round(ms, 4), "algorithmic_bytes_per_elem": bytes_per_elem,
                         "hbm_frac": round(bytes_per_elem * n_params / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        del wts, st1, st2
    except Exception as e:  # the main line must not depend on this leg
        upd = {"error": str(e)}

    # ---- the same K steps with the residue corrections deferred (adacomp_compress_batch_lazy), one
    #      adacomp_residue_sync at the end, inside the timed region; residues start at zero as above.
    #      Reported beside `value`, never as it: the default path is the eager one. -------------------
    lazy = {}
    try:
        if args.no_batch:
            raise RuntimeError("needs the batched entry point")
        if args.no_lazy_leg:
            raise RuntimeError("skipped (--no-lazy-leg)")
        for r in residue:
            r.zero_()
        torch.cuda.synchronize()
        l1, l2 = (torch.cuda.Event(enable_timing=True) for _ in range(2))
        lev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(K)]
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for t in range(K):   # the same three event records per step as the eager loop above
            lev[t][0].record()
            rc = L.adacomp_compress_batch_lazy(layers_c, len(table), n_learners, grad_ptrs[t % n_sets], res_ptrs,
                                               pk_ptrs, bound, ws_p, ws_n, stream)
            if rc:
                raise RuntimeError(f"adacomp_compress_batch_lazy: {rc}")
            lev[t][1].record()
            unpack_all()
            lev[t][2].record()
        l1.record()
        rc = L.adacomp_residue_sync(ws_p, stream)
        if rc:
            raise RuntimeError(f"adacomp_residue_sync: {rc}")
        l2.record()
        torch.cuda.synchronize()
        lazy_ms = (time.perf_counter() - t1) * 1e3 / K
        lazy = {"value": round(grad_bytes_per_step / (lazy_ms * 1e-3) / 1e9, 2), "unit": "GB/s",
                "ms_per_step": round(lazy_ms, 4), "sync_ms": round(l1.elapsed_time(l2), 4),
                "compress_ms_per_step": round(sum(lev[t][0].elapsed_time(lev[t][1]) for t in range(K)) / K, 4),
                "unpack_ms_per_step": round(sum(lev[t][1].elapsed_time(lev[t][2]) for t in range(K)) / K, 4),
                "steps": K, "syncs_in_timed_region": 1, "vs_eager": round(ms_per_step / lazy_ms, 4)}
    except Exception as e:  # the main line must not depend on this leg
        L.adacomp_residue_sync(ws_p, stream)
        torch.cuda.synchronize()
        lazy = {"error": str(e)}

    # ---- CPU oracle on a bounded sample ----------------------------------------------------------------
    cpu = None
    parity = None
    if not args.no_cpu_baseline:
        import oracle
        orc = oracle.Oracle()
        # as many learners of step 0 as fit in about 12 s of single-thread oracle time (at least
        # 2), then one unpack of their packets: the call mix of one GPU step, on fewer learners
        budget_s, n_cpu, pk, dt = 12.0, 0, [], 0.0
        while n_cpu < n_learners and (n_cpu < 2 or dt < budget_s):
            g_host = grads[n_cpu].cpu().numpy()
            r_host = np.zeros(n_total, np.float32)
            t1 = time.perf_counter()
            pk.append(orc.compress(table, g_host, r_host))
            dt += time.perf_counter() - t1
            n_cpu += 1
        t1 = time.perf_counter()
        orc.unpack_accumulate(table, pk, n_total)
        dt += time.perf_counter() - t1
        cpu = {"value": round(n_cpu * 4 * n_params / dt / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": f"{n_cpu} learner(s) x 1 step of {wl.name} (compress each, then one unpack of "
                         f"{n_cpu} packets), single thread, {dt:.1f}s of oracle time"}
        # the same oracle with one learner per host thread (learners are independent; the oracle itself
        # stays single-threaded), then the one unpack: what the host's cores give on the same step
        from concurrent.futures import ThreadPoolExecutor
        n_thr = min(n_learners, len(os.sched_getaffinity(0)), 16)
        hosts = [(grads[k].cpu().numpy(), np.zeros(n_total, np.float32)) for k in range(n_learners)]
        t1 = time.perf_counter()
        with ThreadPoolExecutor(n_thr) as pool:
            pk = list(pool.map(lambda gr: orc.compress(table, gr[0], gr[1]), hosts))
        orc.unpack_accumulate(table, pk, n_total)
        dt_all = time.perf_counter() - t1
        cpu["all_cores"] = {"value": round(n_learners * 4 * n_params / dt_all / 1e9, 4), "unit": "GB/s", "cores": n_thr,
                            "sample": f"{n_learners} learner(s) x 1 step, one learner per thread, then one unpack, {dt_all:.1f}s"}
        # ---- the run checks itself: step 0 from zero residues through the calls that were timed, every
        #      packet, every residue and the dense sum against what the oracle has just computed -------
        sum_want = orc.unpack_accumulate(table, pk, n_total)
        for r in residue:
            r.zero_()
        compress_all(0)
        unpack_all()
        torch.cuda.synchronize()
        mask = np.zeros(n_total, bool)
        for off, n, _ in table:
            mask[off:off + n] = True
        bad = []
        for k in range(n_learners):
            got = packets[k][:pk[k].size].cpu().numpy()
            if not np.array_equal(got, pk[k]):
                bad.append(f"packet {k}")
            if not np.array_equal(residue[k].cpu().numpy()[mask].view(np.uint32), hosts[k][1][mask].view(np.uint32)):
                bad.append(f"residue {k}")
        if not np.array_equal(dense.cpu().numpy()[mask].view(np.uint32), sum_want[mask].view(np.uint32)):
            bad.append("dense sum")
        parity = {"against": "oracle", "step": 0, "packets": n_learners, "residues": n_learners, "dense_sum": True,
                  "bit_equal": not bad}
        if bad:
            log("PARITY FAILURE against the oracle: " + ", ".join(bad))
        del hosts, pk, sum_want

    # ---- the other four configurations, each as configured (its learners, its number of steps, from
    #      zero residues, one batched compress call and one unpack per step) ---------------------------
    per_config = None
    if args.workload == 5 and not args.no_per_config and not args.graph and not args.no_batch:
        A.adacomp_workspace_release(ws)
        del grads, residue, packets, dense, ws
        torch.cuda.empty_cache()
        per_config = {}
        for idx in (1, 2, 3, 4):
            try:
                per_config[W.workload(idx).name] = small_config(W.workload(idx), dev, threads, L, binding, A, W, torch, ctypes)
            except Exception as e:  # the main line must not depend on this leg
                per_config[W.workload(idx).name] = {"error": str(e)}

    out = {
        "metric": "GB/s gradient compressed+unpacked", "value": round(value, 2), "unit": "GB/s",
        "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name} (configuration {wl.index}): {len(table)} layers, {n_params} fp32 elements, "
                               f"L_T {sorted(set(l[2] for l in table))}, {n_learners} simulated learners, residues start at zero",
                   "n_learners": n_learners, "n_elems": n_params, "dist": wl.dist, "seed": 0,
                   "gradient_buffers": n_buf, "fresh_gradient_per_learner_and_step": fresh,
                   "compress_call": "adacomp_compress" if args.no_batch else "adacomp_compress_batch",
                   "launch": "hip_graph_replay" if args.graph else "direct"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "parity_checked": parity,
        "per_config": per_config,
        "hbm_frac_step_algorithmic": round(step_frac, 4), "device_copy_GBs": round(copy_gbs, 1),
        "device_triad_GBs": round(ceilings["triad"], 1), "device_triad_GBs_by_resident_workgroups": triad_by_resident,
        "device_fill_GBs": round(ceilings["fill"], 1),
        "compress_ms_per_step": None if graph is not None else round(compress_ms, 4),
        "unpack_ms_per_step": None if graph is not None else round(unpack_ms, 4),
        "unpack_update": upd,
        "lazy_residue": lazy,
        "compression": {"paper_accounting": round(ratio_paper, 2), "wire": round(ratio_wire, 2),
                        "selected_per_learner_last_step": n_sel // n_learners,
                        "packet_bytes_mean_last_step": int(packet_bytes_mean),
                        "paper_context": "~40x conv / ~200x FC-LSTM on trained gradients"},
    }
    print(json.dumps(out), flush=True)
    if parity is not None and not parity["bit_equal"]:
        sys.exit("bench.py: the timed path's output differs from the oracle's (see parity_checked)")


if __name__ == "__main__":
    main()
