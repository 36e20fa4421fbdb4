#!/usr/bin/env python3
"""Benchmark of the KNN-softmax hot path on one MI355X.

A "step" is one pass of the whole path over one synthetic batch: active-class selection, logits GEMM
(with the row gather), softmax / cross-entropy / logit gradient, dX and dW GEMMs, and the weight update
(knn_softmax_fwd_bwd_update: one call).  The KNN graph is rebuilt once before the loop (knn_graph_build, the
once-per-epoch stage) and timed separately.

Prints ONE JSON line on stdout: whole-job samples/s of the headline workload, the roofline figure of the dominant
kernel (from HIP events recorded around every stage), the two measured peaks of the chip (pure-MFMA loop, streaming
copy) with fractions against both the nominal and the measured peak, the same step at the cap of the active set
(uniform labels) and on the 1M-class workload next to the full softmax over all classes, and the CPU oracle timed on
the host cores on the same inputs.  Everything else goes to stderr.
"""
from __future__ import annotations

import argparse
import ctypes as ct
import json
import os
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

PHASES = ["select", "logits_gemm", "row_stats", "logit_grad", "dx_gemm", "dx_reduce", "dw_gemm", "apply"]

TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "bench_shard390k_hbm_traffic.txt")
# stage of the step -> kernel whose line of the profile gives the stage's HBM traffic per launch
TRAFFIC_KERNEL = {"logits_gemm": "sm_fused_soe_kernel", "dx_gemm": "dx_partial_async_kernel", "dw_gemm": "dw_async_kernel"}


def profiled_traffic(path=TRAFFIC_PROFILE):
    """HBM bytes per launch of the step's kernels, read from the committed rocprofv3 summary (column 'scaled MB' =
    FETCH_SIZE x its calibration factor + WRITE_SIZE; workload shard390k, unit-rows mode, update inside the dW kernel).
    Returns {stage: bytes} (empty when the file is not there)."""
    out = {}
    try:
        lines = open(path).read().splitlines()
    except OSError:
        return out
    for stage, kernel in TRAFFIC_KERNEL.items():
        for ln in lines:
            if ln.startswith(kernel):
                out[stage] = float(ln.split()[-1]) * 1e6
                break
    return out


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class HipEvents:
    """hipEvent_t handles through the HIP runtime already loaded by torch."""

    def __init__(self):
        self.hip = ct.CDLL("libamdhip64.so")
        self.hip.hipEventElapsedTime.argtypes = [ct.POINTER(ct.c_float), ct.c_void_p, ct.c_void_p]

    def create(self, n):
        evs = (ct.c_void_p * n)()
        for k in range(n):
            e = ct.c_void_p()
            rc = self.hip.hipEventCreate(ct.byref(e))
            assert rc == 0, f"hipEventCreate -> {rc}"
            evs[k] = e
        return evs

    def record(self, ev, stream):
        rc = self.hip.hipEventRecord(ct.c_void_p(ev), ct.c_void_p(stream))
        assert rc == 0, f"hipEventRecord -> {rc}"

    def elapsed_ms(self, a, b):
        ms = ct.c_float()
        rc = self.hip.hipEventElapsedTime(ct.byref(ms), ct.c_void_p(a), ct.c_void_p(b))
        assert rc == 0, f"hipEventElapsedTime -> {rc}"
        return float(ms.value)


def make_inputs(cfg, log_fn=log):
    import synth
    t = time.time()
    W, X = synth.make_WX(cfg)
    y = synth.make_labels(cfg)
    log_fn(f"[bench] inputs: C={cfg['C']} D={cfg['D']} B={cfg['B']} K={cfg['K']} M={cfg['M']} labels={cfg['labels']} "
           f"({time.time() - t:.1f}s host generation)")
    return W, X, y


def arithmetic_graph(C, K):
    """K distinct ids per class, none equal to the class: neighbour lists for runs that do not need true neighbours."""
    c = np.arange(C, dtype=np.int64)[:, None]
    k = np.arange(K, dtype=np.int64)[None, :]
    return ((c + 1 + (c * 2654435761 + k * 40503) % (C - 1)) % C).astype(np.int32)


def oracle_graph_for_labels(orc, W, y, cfg):
    """Neighbour lists for the oracle: exact brute force for the rows the selection reads (the labels), a
    synthetic filler elsewhere (never read).  Returns (G, distinct rows, their lists, seconds)."""
    rows = np.unique(y).astype(np.int32)
    t = time.time()
    lists, _ = orc.graph_bruteforce(W, cfg["K"], rows)
    dt = time.time() - t
    G = np.empty((cfg["C"], cfg["K"]), dtype=np.int32)
    G[:] = (np.arange(cfg["C"], dtype=np.int64)[:, None] + 1 + np.arange(cfg["K"])[None, :]) % cfg["C"]
    G[rows] = lists
    return G, rows, lists, dt


def phase_model(cfg, A, unit_rows, fused_update=False):
    """Algorithmic flops / bytes per launch of each stage at A active classes."""
    B, D = cfg["B"], cfg["D"]
    gemm = 2.0 * B * A * D
    return {
        "select": dict(bound="latency"),
        # unit rows: the only sweep (logits -> exponentials stored transposed + their sums); otherwise
        # logits + per-slab softmax statistics, nothing stored
        "logits_gemm": dict(bound="mfma", flops=gemm),
        "row_stats": dict(bound="latency"),                  # merge of the per-slab sums, loss, loss mean
        # logits again -> logit gradient (stored transposed); no such sweep with unit rows
        "logit_grad": dict(bound="latency") if unit_rows else dict(bound="mfma", flops=gemm),
        "dx_gemm": dict(bound="mfma", flops=gemm),
        "dx_reduce": dict(bound="latency"),                  # nothing launched here: the reduction rides with dw_gemm
        "dw_gemm": dict(bound="mfma", flops=gemm),
        # the stand-alone update; nothing is launched here when the update runs inside the dW kernel
        "apply": dict(bound="latency") if fused_update else dict(bound="hbm", bytes=A * D * (4.0 + 4.0 + 4.0 + 2.0)),
    }


def measure_peaks(ks, hev, stream, torch):
    """The two ceilings as this chip sustains them: a loop of independent bf16 MFMAs on registers, a streaming copy."""
    L = ks.lib()
    ev = hev.create(2)
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    wgs, iters = 2 * n_cu, 4000
    out = torch.empty(wgs * 256, dtype=torch.float32, device="cuda")
    flops = ct.c_double(0.0)
    best_mfma = 0.0
    for rep in range(3):
        hev.record(ev[0], stream)
        rc = L.ks_peak_mfma(ct.c_void_p(out.data_ptr()), ct.c_int(wgs), ct.c_int(iters), ct.byref(flops), ct.c_void_p(stream))
        assert rc == 0, rc
        hev.record(ev[1], stream)
        torch.cuda.synchronize()
        if rep:
            best_mfma = max(best_mfma, flops.value / (hev.elapsed_ms(ev[0], ev[1]) * 1e-3) / 1e12)
    nbytes = 1 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    src.zero_()
    best_copy = 0.0
    for rep in range(4):
        hev.record(ev[0], stream)
        rc = L.ks_peak_copy(ct.c_void_p(src.data_ptr()), ct.c_void_p(dst.data_ptr()), ct.c_size_t(nbytes), ct.c_int(16 * n_cu),
                            ct.c_void_p(stream))
        assert rc == 0, rc
        hev.record(ev[1], stream)
        torch.cuda.synchronize()
        if rep:
            best_copy = max(best_copy, 2.0 * nbytes / (hev.elapsed_ms(ev[0], ev[1]) * 1e-3) / 1e9)
    del src, dst, out
    return dict(mfma_loop_tflops=round(best_mfma, 1), stream_copy_gbs=round(best_copy, 1),
                what="pure v_mfma_f32_32x32x16_bf16 loop on registers, 2 workgroups of 4 wavefronts per compute unit; "
                     "copy of 1 GiB with 16-byte loads and stores (read + written bytes)")


class StepRunner:
    """One workload's buffers and the three timed loops over its step."""

    def __init__(self, ks, torch, hev, cfg, W, X, y, graph, unit_rows, fused_update, W_bf=None, W_master=None,
                 next_inside=False):
        """next_inside: a step is ONE call of knn_softmax_fwd_bwd_update_selected_next -- forward, backward and weight
        update of this batch on the list the previous call left, and Algorithm 1 for the next batch in the same launches
        (every step still runs every stage once).  Otherwise ONE call of knn_softmax_fwd_bwd_update."""
        self.ks, self.torch, self.hev, self.cfg = ks, torch, hev, cfg
        C, D, B, K, M = cfg["C"], cfg["D"], cfg["B"], cfg["K"], cfg["M"]
        self.scale, self.grad_scale = cfg["scale"], 128.0
        self.alpha = -0.05 / self.grad_scale
        self.unit_rows, self.fused = unit_rows, fused_update
        self.W_bf = W_bf if W_bf is not None else torch.from_numpy(W).cuda().to(torch.bfloat16)
        self.W_master = W_master if W_master is not None else torch.from_numpy(W).cuda()
        self.X_bf = torch.from_numpy(X).cuda().to(torch.bfloat16)
        self.labels = torch.from_numpy(y).cuda()
        self.graph = graph
        self.stream = torch.cuda.current_stream().cuda_stream
        self.ws = torch.empty(ks.knn_softmax_workspace(C, D, B, K, M), dtype=torch.uint8, device="cuda")
        self.out = ks.knn_softmax_fwd_bwd(self.W_bf, self.X_bf, self.labels, graph, M, self.scale, self.grad_scale, ws=self.ws,
                                          unit_rows=unit_rows)
        torch.cuda.synchronize()
        assert int(self.out["dev_status"].item()) == 0
        self.A = int(self.out["n_active"].item())
        self.out_fused = dict(self.out)
        self.out_fused["dW_active"] = None      # the fused step does not store the gradient rows
        self.next_inside = bool(next_inside and fused_update)
        if self.next_inside:
            self.ws_next = torch.empty(ks.knn_softmax_selected_next_workspace(C, D, B, K, M), dtype=torch.uint8, device="cuda")
            # the list of the first batch; every call reads one set of buffers in place (they are the library's own
            # output: KS_FLAG_TRUSTED_LIST) and leaves the next batch's list in the other
            self.sel = {k: self.out[k].clone() for k in ("active_idx", "n_active", "target_pos")}
            self.sel_other = {k: self.out[k].clone() for k in ("active_idx", "n_active", "target_pos")}
            self.out_next = {k: self.out[k] for k in ("loss_per_sample", "loss_mean", "dX", "dev_status")}
            self.out_next["dW_active"] = None

    def first_step_copy(self):
        first = {k: self.out[k].clone() for k in ("active_idx", "target_pos", "loss_per_sample", "loss_mean", "dX")}
        first["dW_active"] = self.out["dW_active"][:self.A].clone()
        return first

    def step(self, ev=None):
        ks, cfg, o = self.ks, self.cfg, self.out
        C, D, B, K, M = cfg["C"], cfg["D"], cfg["B"], cfg["K"], cfg["M"]
        if ev is None and self.next_inside:
            ks.knn_softmax_fwd_bwd_update_selected_next(self.W_master, self.W_bf, self.X_bf, self.sel["active_idx"],
                                                        self.sel["n_active"], self.sel["target_pos"], self.labels, self.graph,
                                                        self.scale, self.grad_scale, self.alpha, next_out=self.sel_other,
                                                        out=self.out_next, ws=self.ws_next, unit_rows=self.unit_rows,
                                                        trusted_list=True)
            self.sel, self.sel_other = self.sel_other, self.sel
            return
        if ev is None and self.fused:
            ks.knn_softmax_fwd_bwd_update(self.W_master, self.W_bf, self.X_bf, self.labels, self.graph, M, self.scale,
                                          self.grad_scale, self.alpha, out=self.out_fused, ws=self.ws, unit_rows=self.unit_rows)
            return
        if ev is None:
            ks.knn_softmax_fwd_bwd(self.W_bf, self.X_bf, self.labels, self.graph, M, self.scale, self.grad_scale, out=o,
                                   ws=self.ws, unit_rows=self.unit_rows)
        else:
            rc = ks.lib().knn_softmax_fwd_bwd_profiled(
                ct.c_void_p(self.W_master.data_ptr() if self.fused else 0), ct.c_void_p(self.W_bf.data_ptr()),
                ct.c_void_p(self.X_bf.data_ptr()), ct.c_void_p(self.labels.data_ptr()),
                ct.c_void_p(self.graph.data_ptr()), ct.c_int64(C), ct.c_int(D), ct.c_int(B), ct.c_int(K), ct.c_int(M),
                ct.c_float(self.scale), ct.c_float(self.grad_scale), ct.c_float(self.alpha),
                ct.c_uint32(1 if self.unit_rows else 0), ct.c_void_p(o["active_idx"].data_ptr()),
                ct.c_void_p(o["n_active"].data_ptr()), ct.c_void_p(o["target_pos"].data_ptr()),
                ct.c_void_p(o["loss_per_sample"].data_ptr()), ct.c_void_p(o["loss_mean"].data_ptr()),
                ct.c_void_p(o["dX"].data_ptr()), ct.c_void_p(0 if self.fused else o["dW_active"].data_ptr()),
                ct.c_void_p(self.ws.data_ptr()), ct.c_size_t(self.ws.numel()), ct.c_void_p(o["dev_status"].data_ptr()),
                ct.c_void_p(self.stream), ev, ct.c_int(8))
            assert rc == 0, rc
        if not self.fused:
            ks.apply_weight_grad(self.W_master, self.W_bf, o["active_idx"], o["n_active"], o["dW_active"], self.alpha,
                                 idx_sorted_unique=True, ws=self.ws, dev_status=o["dev_status"])
        if ev is not None:
            self.hev.record(ev[8], self.stream)

    def run(self, steps, warmup, with_stages=True):
        """(ms per step by the wall clock over `steps` steps, median ms per step between HIP events recorded at the
        step boundaries, stage times in microseconds or None)."""
        torch, hev = self.torch, self.hev
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        # timed region: K steps, nothing but the library's own launches on the stream
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        ms_wall = (time.perf_counter() - t0) * 1e3 / steps
        assert int(self.out["dev_status"].item()) == 0
        # the same K steps with one HIP event at every step boundary: median of the K differences
        bev = hev.create(steps + 1)
        hev.record(bev[0], self.stream)
        for s in range(steps):
            self.step()
            hev.record(bev[s + 1], self.stream)
        torch.cuda.synchronize()
        ms_median = statistics.median(hev.elapsed_ms(bev[s], bev[s + 1]) for s in range(steps))
        dur = None
        if with_stages:
            # and with a HIP event at every stage boundary (the records cost a few microseconds each, which is why
            # they are kept out of the regions above)
            evs = [hev.create(9) for _ in range(steps)]
            for s in range(steps):
                self.step(evs[s])
            torch.cuda.synchronize()
            assert int(self.out["dev_status"].item()) == 0
            dur = {p: statistics.median(hev.elapsed_ms(ev[k], ev[k + 1]) for ev in evs) * 1e3 for k, p in enumerate(PHASES)}
        return ms_wall, ms_median, dur


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="shard390k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-parity", action="store_true")
    ap.add_argument("--headline-only", action="store_true",
                    help="only the headline step (no other workloads, layers or peaks): used for the profiles")
    ap.add_argument("--serial", action="store_true",
                    help="headline = the one-call step that selects its own batch first (default: the next batch's selection "
                         "rides along with the step)")
    ap.add_argument("--separate-update", action="store_true",
                    help="run the weight update as a call of its own (apply_weight_grad) instead of knn_softmax_fwd_bwd_update")
    ap.add_argument("--general-rows", action="store_true",
                    help="do not tell the library that the rows are L2-normalised (two-sweep softmax)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus must be 1")
        sys.exit(2)

    import torch
    import synth
    import paper_2102_06025_amd as ks

    ks.lib()  # fails loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    cfg = dict(synth.CONFIGS[args.workload])
    C, D, B, K, M, scale = cfg["C"], cfg["D"], cfg["B"], cfg["K"], cfg["M"], cfg["scale"]

    W, X, y = make_inputs(cfg)
    W_bf = torch.from_numpy(W).cuda().to(torch.bfloat16)
    W_master = torch.from_numpy(W).cuda()
    stream = torch.cuda.current_stream().cuda_stream
    hev = HipEvents()
    L = ks.lib()

    # ---- the chip's own ceilings ------------------------------------------------------------------------
    peaks = None
    if not args.headline_only:
        peaks = measure_peaks(ks, hev, stream, torch)
        log(f"[bench] measured peaks: {peaks['mfma_loop_tflops']:.0f} TFLOP/s in a pure MFMA loop "
            f"({peaks['mfma_loop_tflops'] / PEAK_BF16_TFLOPS:.0%} of nominal), {peaks['stream_copy_gbs']:.0f} GB/s in a streaming copy "
            f"({peaks['stream_copy_gbs'] / PEAK_HBM_GBS:.0%} of nominal)")

    def fracs(achieved, nominal, measured):
        d = dict(frac=round(achieved / nominal, 4))
        if measured:
            d["frac_of_measured_peak"] = round(achieved / measured, 4)
        return d

    # ---- graph rebuild (once per epoch in the paper; timed on its own) -------------------------------
    g_ws = torch.empty(ks.knn_graph_build_workspace(C, D, K, 0), dtype=torch.uint8, device="cuda")
    graph = torch.empty((C, K), dtype=torch.int32, device="cuda")
    gev = hev.create(2)
    graph_ms = []
    for _ in range(2):
        hev.record(gev[0], stream)
        ks.knn_graph_build(W_bf, K, graph=graph, ws=g_ws)
        hev.record(gev[1], stream)
        torch.cuda.synchronize()
        graph_ms.append(hev.elapsed_ms(gev[0], gev[1]))
    del g_ws
    graph_best = min(graph_ms)
    graph_tflops = 2.0 * C * C * D / (graph_best * 1e-3) / 1e12
    log(f"[bench] knn_graph_build: {graph_best:.1f} ms  ({graph_tflops:.0f} TFLOP/s algorithmic, "
        f"{graph_tflops / PEAK_BF16_TFLOPS:.1%} of bf16 peak)")

    # ---- the headline step ----------------------------------------------------------------------------------
    # the synthetic rows are L2-normalised, as the paper's are: the library may rely on it
    unit_rows = not args.general_rows
    fused_update = not args.separate_update
    # The headline loop is the training loop's: one library call per step, which runs forward, backward and weight update
    # of batch n and Algorithm 1 for batch n + 1 (whose labels a data loader has early) in the same launches.  --serial
    # times the one-call step that selects its own batch first (reported beside it in any case).
    next_inside = fused_update and not args.serial
    run = StepRunner(ks, torch, hev, cfg, W, X, y, graph, unit_rows, fused_update, W_bf=W_bf, W_master=W_master,
                     next_inside=next_inside)
    A = run.A
    log(f"[bench] active classes A={A} of M={M}")
    first = run.first_step_copy()
    out, ws = run.out, run.ws
    X_bf, labels = run.X_bf, run.labels
    grad_scale, alpha = run.grad_scale, run.alpha
    ms_per_step, ms_median, dur = run.run(args.steps, args.warmup)
    value = B / (ms_per_step * 1e-3)
    ms_serial = ms_per_step
    if next_inside:
        assert torch.equal(run.sel["active_idx"], run.out["active_idx"]) and torch.equal(run.sel["target_pos"], run.out["target_pos"])
        run.next_inside = False
        ms_serial, _, _ = run.run(args.steps, args.warmup, with_stages=False)
        run.next_inside = True
        log(f"[bench] step with the next batch's selection inside: {ms_per_step:.4f} ms; one-call step that selects first: {ms_serial:.4f} ms")

    mfma_peak = peaks["mfma_loop_tflops"] if peaks else None
    copy_peak = peaks["stream_copy_gbs"] if peaks else None
    model = phase_model(cfg, A, unit_rows, fused_update)
    phases = {}
    for p in PHASES:
        m = model[p]
        e = dict(us=round(dur[p], 2), bound=m["bound"])
        if "flops" in m:
            e["tflops"] = round(m["flops"] / (dur[p] * 1e-6) / 1e12, 1)
            e.update(fracs(e["tflops"], PEAK_BF16_TFLOPS, mfma_peak))
        elif "bytes" in m:
            e["gbs"] = round(m["bytes"] / (dur[p] * 1e-6) / 1e9, 1)
            e.update(fracs(e["gbs"], PEAK_HBM_GBS, copy_peak))
        phases[p] = e
    if next_inside:
        phases["select"]["note"] = ("stage times are those of the one-call step; in the headline loop the selection (of the next "
                                    "batch) runs inside the dx_gemm and dw_gemm launches and adds nothing to the step")
    log("[bench] stage times (us, medians): " + ", ".join(f"{p}={phases[p]['us']}" for p in PHASES))
    traffic_all = profiled_traffic() if (unit_rows and fused_update and args.workload == "shard390k") else {}
    dom = max((p for p in PHASES if model[p]["bound"] in ("mfma", "hbm")), key=lambda p: dur[p])
    traffic = traffic_all.get(dom)
    if model[dom]["bound"] == "mfma":
        roofline = dict(bound="mfma", achieved=phases[dom]["tflops"], peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                        frac=phases[dom]["frac"], traffic=traffic, kernel=dom,
                        traffic_source=os.path.relpath(TRAFFIC_PROFILE, ROOT) if traffic else None)
        if mfma_peak:
            roofline.update(measured_peak=mfma_peak, frac_of_measured_peak=phases[dom]["frac_of_measured_peak"])
        if dom == "dw_gemm" and fused_update:
            # this launch is two things: the dW contraction (the flops counted above) and the weight update of the
            # active rows in its epilogue, which is HBM work; both against their own peaks, one after the other
            upd_bytes = A * D * (4.0 + 4.0 + 2.0)
            t_roof = model[dom]["flops"] / (PEAK_BF16_TFLOPS * 1e12) + upd_bytes / (PEAK_HBM_GBS * 1e9)
            roofline.update(kernel="dw_gemm + weight update (one launch)", update_bytes=upd_bytes,
                            frac_of_two_phase_roofline=round(t_roof / (dur[dom] * 1e-6), 4),
                            runner_up=dict(kernel="logits_gemm", bound="mfma", achieved=phases["logits_gemm"]["tflops"],
                                           frac=phases["logits_gemm"]["frac"], us=phases["logits_gemm"]["us"],
                                           traffic=traffic_all.get("logits_gemm")))
            # Which roofline binds the launch?  Its algorithmic bytes: the logit gradient (A x B bf16) and X / sum (B x D
            # bf16) read, the fp32 rows of the active classes read and written, their 16-bit copies written, dX (B x D
            # fp32) written.  At the nominal peaks they take longer than its flops: the launch is bound by HBM, and that
            # is the figure reported; the matrix-core view stays beside it.
            launch_bytes = A * B * 2.0 + B * D * 2.0 + upd_bytes + B * D * 4.0
            if launch_bytes / (PEAK_HBM_GBS * 1e9) > model[dom]["flops"] / (PEAK_BF16_TFLOPS * 1e12):
                as_mfma = dict(achieved=roofline["achieved"], peak=PEAK_BF16_TFLOPS, unit="TFLOP/s", frac=roofline["frac"],
                               measured_peak=roofline.get("measured_peak"),
                               frac_of_measured_peak=roofline.get("frac_of_measured_peak"))
                gbs = launch_bytes / (dur[dom] * 1e-6) / 1e9
                roofline.update(bound="hbm", achieved=round(gbs, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                                frac=round(gbs / PEAK_HBM_GBS, 4), algorithmic_bytes=launch_bytes, as_mfma=as_mfma,
                                bound_reason=f"at the nominal peaks the launch's {launch_bytes / 1e6:.1f} MB take "
                                             f"{launch_bytes / (PEAK_HBM_GBS * 1e9) * 1e6:.1f} us and its "
                                             f"{model[dom]['flops'] / 1e9:.1f} GFLOP {model[dom]['flops'] / (PEAK_BF16_TFLOPS * 1e12) * 1e6:.1f} us")
                if copy_peak:
                    roofline.update(measured_peak=copy_peak, frac_of_measured_peak=round(gbs / copy_peak, 4))
    else:
        roofline = dict(bound="hbm", achieved=phases[dom]["gbs"], peak=PEAK_HBM_GBS, unit="GB/s",
                        frac=phases[dom]["frac"], traffic=traffic, kernel=dom)
    # whole step against the matrix peak: all of the path's contractions over its whole duration
    step_flops = sum(m.get("flops", 0.0) for m in model.values())
    whole_step = dict(gflop=round(step_flops / 1e9, 2), tflops=round(step_flops / (ms_per_step * 1e-3) / 1e12, 1))
    whole_step.update(fracs(whole_step["tflops"], PEAK_BF16_TFLOPS, mfma_peak))

    def timed_events(fn, reps, warm=3):
        ev = hev.create(2)
        for _ in range(warm):
            fn()
        hev.record(ev[0], stream)
        for _ in range(reps):
            fn()
        hev.record(ev[1], stream)
        torch.cuda.synchronize()
        return hev.elapsed_ms(ev[0], ev[1]) * 1e3 / reps

    def hbm_entry(us, nbytes):
        gbs = nbytes / (us * 1e-6) / 1e9
        e = dict(us=round(us, 2), bound="hbm", gbs=round(gbs, 1))
        e.update(fracs(gbs, PEAK_HBM_GBS, copy_peak))
        return e

    # ---- the row gather as a kernel of its own (in the step it is fused into the loaders of the contractions):
    # A rows of D bf16 values read and written once
    gather = None
    if not args.headline_only:
        g_out = torch.empty((M, D), dtype=torch.bfloat16, device="cuda")
        g_st = torch.zeros(1, dtype=torch.int32, device="cuda")
        us_g = timed_events(lambda: ks.knn_gather_rows(W_bf, out["active_idx"], out["n_active"], out=g_out, dev_status=g_st), 20)
        gather = hbm_entry(us_g, A * D * 2.0 * 2)
        log(f"[bench] stand-alone gather of the {A} active rows: {gather}")
        del g_out

    # ---- the step when the selection is not on its critical path (Algorithm 1 needs only the labels): (a) the selection
    # given -- made earlier, e.g. while the features of the batch were still being computed; (b) the selection of the
    # NEXT batch on a second stream, one event dependency per step.  The headline figure is the serial one-call step.
    selection_variants = None
    if fused_update and not args.headline_only:
        side = torch.cuda.Stream()
        main_s = torch.cuda.current_stream()
        sel_bufs = [dict(active_idx=torch.empty(M, dtype=torch.int32, device="cuda"),
                         n_active=torch.empty(1, dtype=torch.int32, device="cuda"),
                         target_pos=torch.empty(B, dtype=torch.int32, device="cuda"),
                         ws=torch.empty(ks.knn_select_workspace(C, B, K, M), dtype=torch.uint8, device="cuda")) for _ in range(2)]
        sel_st = torch.zeros(1, dtype=torch.int32, device="cuda")
        ws_sel = torch.empty(ks.knn_softmax_selected_workspace(C, D, B, M), dtype=torch.uint8, device="cuda")
        e_sel = [torch.cuda.Event(), torch.cuda.Event()]
        e_use = [torch.cuda.Event(), torch.cuda.Event()]
        out_sel = None

        def select_on(slot, stream):
            b = sel_bufs[slot]
            rc = ks.lib().knn_select_active(ct.c_void_p(labels.data_ptr()), ct.c_void_p(graph.data_ptr()), ct.c_int64(C),
                                            ct.c_int(B), ct.c_int(K), ct.c_int(M), ct.c_void_p(b["active_idx"].data_ptr()),
                                            ct.c_void_p(b["n_active"].data_ptr()), ct.c_void_p(b["target_pos"].data_ptr()),
                                            ct.c_void_p(b["ws"].data_ptr()), ct.c_size_t(b["ws"].numel()),
                                            ct.c_void_p(sel_st.data_ptr()), ct.c_void_p(stream.cuda_stream))
            assert rc == 0, rc

        def step_selected(slot):
            nonlocal out_sel
            b = sel_bufs[slot]
            out_sel = ks.knn_softmax_fwd_bwd_update_selected(W_master, W_bf, X_bf, b["active_idx"], b["n_active"],
                                                             b["target_pos"], cfg["scale"], grad_scale, alpha,
                                                             out=out_sel, ws=ws_sel, unit_rows=unit_rows)

        def pipelined(n):
            select_on(0, side)
            e_sel[0].record(side)
            for s in range(n):
                slot = s & 1
                main_s.wait_event(e_sel[slot])
                step_selected(slot)
                e_use[slot].record(main_s)
                if s + 1 < n:
                    if s >= 1:
                        side.wait_event(e_use[slot ^ 1])
                    select_on(slot ^ 1, side)
                    e_sel[slot ^ 1].record(side)

        select_on(0, main_s)
        for _ in range(args.warmup):
            step_selected(0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step_selected(0)
        torch.cuda.synchronize()
        ms_given = (time.perf_counter() - t0) * 1e3 / args.steps
        pipelined(args.warmup)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        pipelined(args.steps)
        torch.cuda.synchronize()
        ms_piped = (time.perf_counter() - t0) * 1e3 / args.steps
        assert int(out_sel["dev_status"].item()) == 0 and int(sel_st.item()) == 0
        selection_variants = dict(serial_ms_per_step=round(ms_serial, 4), selection_given_ms_per_step=round(ms_given, 4),
                                  selection_of_next_batch_on_second_stream_ms_per_step=round(ms_piped, 4),
                                  selection_of_next_batch_inside_the_step_ms_per_step=round(ms_per_step, 4) if next_inside else None,
                                  what="serial: knn_softmax_fwd_bwd_update, which selects its own batch first; given / second "
                                       "stream: knn_select_active + knn_softmax_fwd_bwd_update_selected (the second-stream "
                                       "figure includes the cross-stream event dependencies of every step); inside: "
                                       "knn_softmax_fwd_bwd_update_selected_next, the next batch's selection as extra "
                                       "workgroups of the step's dX and dW launches")
        log(f"[bench] selection off the path: given {ms_given:.4f} ms/step, next batch's on a second stream {ms_piped:.4f} "
            f"ms/step (serial {ms_serial:.4f})")
        del sel_bufs, ws_sel

    # ---- the same step at the cap of the active set (uniform labels: about 32.3 k distinct candidates) ----------
    at_the_cap = None
    if args.workload == "shard390k" and not args.headline_only:
        cfg_u = dict(synth.CONFIGS["shard390k_uniform"])
        run_u = StepRunner(ks, torch, hev, cfg_u, W, X, synth.make_labels(cfg_u), graph, unit_rows, fused_update, W_bf=W_bf,
                           W_master=W_master, next_inside=next_inside)
        ms_u, ms_u_med, dur_u = run_u.run(args.steps, args.warmup)
        gemm_u = 2.0 * B * run_u.A * D
        at_the_cap = dict(workload="shard390k_uniform", active_classes=run_u.A, ms_per_step=round(ms_u, 4),
                          ms_per_step_hip_event_median=round(ms_u_med, 4), samples_per_s=round(B / (ms_u * 1e-3), 1),
                          stage_us={p: round(dur_u[p], 2) for p in PHASES},
                          step_tflops=round(3 * gemm_u / (ms_u * 1e-3) / 1e12, 1),
                          step_frac=round(3 * gemm_u / (ms_u * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4))
        log(f"[bench] at the cap (uniform labels): A={run_u.A}, {ms_u:.4f} ms/step")
        del run_u

    normalized_layer = None
    if not args.headline_only:
        # ---- the layer with un-normalised fp32 weights (normalisation inside the layer, Section 3.2.3): the same step
        # with X normalised on the way in, dX projected on the way out and the weight update through the
        # normalisation; timed after the headline region, reported beside it
        inv_norm = torch.empty(C, dtype=torch.float32, device="cuda")
        ks.knn_normalize_rows(W_master, out_bf16=W_bf, out_inv_norm=inv_norm)
        X_raw = torch.from_numpy(X).cuda()
        dX_raw = torch.empty_like(out["dX"])

        def step_normalized():
            ks.knn_normalize_rows(X_raw, want_inv_norm=False, out_bf16=X_bf)
            ks.knn_softmax_fwd_bwd(W_bf, X_bf, labels, graph, M, scale, grad_scale, out=out, ws=ws, unit_rows=True)
            ks.knn_norm_backward_rows(X_raw, out["dX"], out=dX_raw)
            ks.apply_weight_grad_normalized(W_master, W_bf, inv_norm, out["active_idx"], out["n_active"], out["dW_active"],
                                            alpha, idx_sorted_unique=True, ws=ws, dev_status=out["dev_status"])

        for _ in range(args.warmup):
            step_normalized()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(args.steps):
            step_normalized()
        torch.cuda.synchronize()
        ms_norm_step = (time.perf_counter() - t0) * 1e3 / args.steps
        # the same as a training loop runs it: the next batch's selection inside the softmax call (W_master = NULL: the
        # gradient rows are stored for the update through the normalisation), lists read in place, two sets in turn
        nl = [{k_: out[k_].clone() for k_ in ("active_idx", "n_active", "target_pos")} for _ in range(2)]
        nl_ws = torch.empty(ks.knn_softmax_selected_next_workspace(C, D, B, K, M), dtype=torch.uint8, device="cuda")
        nl_out = {k_: out[k_] for k_ in ("loss_per_sample", "loss_mean", "dX", "dW_active", "dev_status")}

        def step_normalized_next():
            a, b = nl
            ks.knn_normalize_rows(X_raw, want_inv_norm=False, out_bf16=X_bf)
            ks.knn_softmax_fwd_bwd_update_selected_next(None, W_bf, X_bf, a["active_idx"], a["n_active"], a["target_pos"], labels,
                                                        graph, scale, grad_scale, 0.0, next_out=b, out=nl_out, ws=nl_ws,
                                                        unit_rows=True, trusted_list=True)
            ks.knn_norm_backward_rows(X_raw, out["dX"], out=dX_raw)
            ks.apply_weight_grad_normalized(W_master, W_bf, inv_norm, a["active_idx"], a["n_active"], out["dW_active"], alpha,
                                            idx_sorted_unique=True, ws=ws, dev_status=out["dev_status"])
            nl.reverse()

        for _ in range(args.warmup):
            step_normalized_next()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(args.steps):
            step_normalized_next()
        torch.cuda.synchronize()
        ms_norm_next = (time.perf_counter() - t0) * 1e3 / args.steps
        del nl_ws
        us_apply_n = timed_events(lambda: ks.apply_weight_grad_normalized(
            W_master, W_bf, inv_norm, out["active_idx"], out["n_active"], out["dW_active"], alpha, idx_sorted_unique=True,
            ws=ws, dev_status=out["dev_status"]), args.steps, warm=0)
        assert int(out["dev_status"].item()) == 0
        normalized_layer = dict(ms_per_step=round(ms_norm_step, 4), samples_per_s=round(B / (ms_norm_step * 1e-3), 1),
                                step="normalize X + select + knn_softmax_fwd_bwd + project dX + apply_weight_grad_normalized",
                                ms_per_step_next_selection_inside=round(ms_norm_next, 4),
                                step_next_selection_inside="normalize X + knn_softmax_fwd_bwd_update_selected_next without update "
                                                           "(selects the next batch inside) + project dX + "
                                                           "apply_weight_grad_normalized",
                                apply_normalized=hbm_entry(us_apply_n, A * (D * (4.0 + 4.0 + 4.0 + 2.0) + 4.0)))
        log(f"[bench] layer with normalisation inside: {ms_norm_step:.4f} ms/step ({ms_norm_next:.4f} with the next selection "
            f"inside), apply_normalized {us_apply_n:.1f} us")

    # ---- this GPU as one node of four (Section 3.2.3): graph compression and selection on the compressed graph,
    # with and without the random fill-up to M (Algorithm 1); integer work, bit-exact against the oracle in the tests
    sharded_node = None
    if args.workload == "shard390k" and not args.headline_only:
        Cg4, c0 = 4 * C, C
        G4 = torch.from_numpy(arithmetic_graph(Cg4, K)).cuda()
        y4 = torch.from_numpy(synth.labels_zipf(cfg["seed"], B, Cg4, 1.1)).cuda()
        counts, offsets, flat, st4 = ks.knn_graph_compress(G4, c0, C)
        c_ws = torch.empty(int(L.knn_graph_compress_workspace(ct.c_int64(Cg4), ct.c_int(K))), dtype=torch.uint8, device="cuda")
        s_ws = torch.empty(ks.knn_select_active_csr_workspace(C, B, K, M), dtype=torch.uint8, device="cuda")

        def compress():
            rc = L.knn_graph_compress(ct.c_void_p(G4.data_ptr()), ct.c_int64(Cg4), ct.c_int(K), ct.c_int64(c0), ct.c_int64(C),
                                      ct.c_void_p(counts.data_ptr()), ct.c_void_p(offsets.data_ptr()),
                                      ct.c_void_p(flat.data_ptr()), ct.c_int64(flat.numel()), ct.c_void_p(c_ws.data_ptr()),
                                      ct.c_size_t(c_ws.numel()), ct.c_void_p(st4.data_ptr()), ct.c_void_p(stream))
            assert rc == 0, rc

        us_compress = timed_events(compress, 10, warm=1)
        us_sel = timed_events(lambda: ks.knn_select_active_csr(y4, counts, offsets, flat, c0, C, K, M, ws=s_ws, dev_status=st4), 20,
                              warm=1)
        us_sel_pad = timed_events(lambda: ks.knn_select_active_csr(y4, counts, offsets, flat, c0, C, K, M, pad_random=True,
                                                                   pad_seed=1, ws=s_ws, dev_status=st4), 20, warm=1)
        o4 = ks.knn_select_active_csr(y4, counts, offsets, flat, c0, C, K, M, ws=s_ws, dev_status=st4)
        torch.cuda.synchronize()
        assert int(st4.item()) == 0
        # the node's whole step with the softmax split over the nodes (Section 3.1 steps 3-5): selection with fill-up,
        # statistics out, [exchange: here the node's own statistics times a constant stand in for the other nodes'],
        # gradients from the combined statistics, weight update
        sp_ws = torch.empty(ks.knn_softmax_split_workspace(C, D, B, M), dtype=torch.uint8, device="cuda")
        ks.knn_normalize_rows(W_master, out_bf16=W_bf, out_inv_norm=inv_norm)

        def node_step(pad):
            sel = ks.knn_select_active_csr(y4, counts, offsets, flat, c0, C, K, M, pad_random=pad, pad_seed=7, ws=s_ws,
                                           dev_status=st4)
            s1 = ks.knn_softmax_fwd_stats(W_bf, X_bf, sel["active_idx"], sel["n_active"], sel["target_pos"], scale,
                                          unit_rows=True, ws=sp_ws, dev_status=st4)
            s1["row_sumexp"].mul_(4.0)      # "all-reduce": four nodes with equal sums (the reference is the same on all)
            s2 = ks.knn_softmax_bwd_from_stats(W_bf, X_bf, sel["active_idx"], sel["n_active"], sel["target_pos"], s1["row_max"],
                                               s1["row_sumexp"], s1["target_logit"], scale, grad_scale, sp_ws,
                                               unit_rows=True, dev_status=st4)
            ks.apply_weight_grad_normalized(W_master, W_bf, inv_norm, sel["active_idx"], sel["n_active"], s2["dW_active"],
                                            alpha, idx_sorted_unique=True, ws=ws, dev_status=st4)
            return sel

        # the same step as a training loop runs it: the next batch's selection inside the second call's launches, the
        # list read in place from the buffers the previous step wrote (two sets in turn)
        spn_ws = torch.empty(ks.knn_softmax_split_next_workspace(C, D, B, K, M), dtype=torch.uint8, device="cuda")
        node_lists = {}

        def node_step_next(pad):
            if pad not in node_lists:
                o = ks.knn_select_active_csr(y4, counts, offsets, flat, c0, C, K, M, pad_random=pad, pad_seed=7, ws=s_ws,
                                             dev_status=st4)
                first = {k_: o[k_] for k_ in ("active_idx", "n_active", "n_found", "target_pos")}
                node_lists[pad] = [first, {k_: torch.empty_like(v) for k_, v in first.items()}]
            a, b = node_lists[pad]
            s1 = ks.knn_softmax_fwd_stats(W_bf, X_bf, a["active_idx"], a["n_active"], a["target_pos"], scale, unit_rows=True,
                                          ws=spn_ws, dev_status=st4, trusted_list=True)
            s1["row_sumexp"].mul_(4.0)
            s2, _ = ks.knn_softmax_bwd_from_stats_next(W_bf, X_bf, a["active_idx"], a["n_active"], a["target_pos"], s1["row_max"],
                                                       s1["row_sumexp"], s1["target_logit"], scale, grad_scale, spn_ws, y4, counts,
                                                       offsets, flat, c0, K, next_out=b, pad_random=pad, pad_seed=7,
                                                       unit_rows=True, trusted_list=True, dev_status=st4)
            ks.apply_weight_grad_normalized(W_master, W_bf, inv_norm, a["active_idx"], a["n_active"], s2["dW_active"], alpha,
                                            idx_sorted_unique=True, ws=ws, dev_status=st4)
            node_lists[pad] = [b, a]

        def wall(fn, reps):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / reps

        ms_node = wall(lambda: node_step(False), args.steps)
        ms_node_pad = wall(lambda: node_step(True), args.steps)
        ms_node_next = wall(lambda: node_step_next(False), args.steps)
        ms_node_next_pad = wall(lambda: node_step_next(True), args.steps)
        n_act4 = int(node_step(False)["n_active"].item())
        torch.cuda.synchronize()
        assert int(st4.item()) == 0
        # algorithmic traffic of the compression: the dense graph read once, counts, offsets and lists written
        bytes_c = Cg4 * K * 4.0 + flat.numel() * 4.0 + Cg4 * (4.0 + 8.0)
        sharded_node = dict(problem=f"Cg={Cg4} classes on 4 nodes, this node owns [{c0}, {c0 + C}); K={K}, global batch {B}",
                            compressed_entries=int(flat.numel()), classes_found=int(o4["n_found"].item()),
                            graph_compress=hbm_entry(us_compress, bytes_c),
                            select_csr_us=round(us_sel, 2), select_csr_with_fill_up_us=round(us_sel_pad, 2),
                            node_step=dict(what="select_csr + fwd_stats + exchange stand-in + bwd_from_stats + "
                                                "apply_weight_grad_normalized, one-sweep softmax",
                                           ms_per_step=round(ms_node, 4), active_classes=n_act4,
                                           ms_per_step_filled_to_M=round(ms_node_pad, 4),
                                           next_selection_inside=dict(
                                               what="fwd_stats + exchange stand-in + knn_softmax_bwd_from_stats_next (the next "
                                                    "batch's select_csr inside its launches, lists read in place) + "
                                                    "apply_weight_grad_normalized",
                                               ms_per_step=round(ms_node_next, 4),
                                               ms_per_step_filled_to_M=round(ms_node_next_pad, 4))))
        log(f"[bench] one node of four: compress {us_compress:.0f} us, select {us_sel:.1f} us, with fill-up {us_sel_pad:.1f} us; "
            f"node step {ms_node:.4f} ms (A={n_act4}), filled to M {ms_node_pad:.4f} ms; with the next selection inside "
            f"{ms_node_next:.4f} / {ms_node_next_pad:.4f} ms")
        del G4, sp_ws, spn_ws, node_lists, c_ws, counts, offsets, flat

    # ---- second workload (Section 3.3.2): layer-wise top-k selection over the gradient set of a ResNet-50, 99.9 %
    # sparsity, all 161 tensors in one call; HBM-bound by its algorithmic bytes: every gradient is read once
    grad_topk = None
    if args.workload == "shard390k" and not args.headline_only:
        sizes = synth.resnet50_tensor_sizes()
        g_host, offs = synth.grad_tensor_set(cfg["seed"], sizes)
        kk = synth.topk_counts(sizes)
        plan = ks.grad_topk_plan(offs, kk)
        g_dev = torch.from_numpy(g_host).cuda()
        t_idx = torch.empty(plan.n_out, dtype=torch.int32, device="cuda")
        t_val = torch.empty(plan.n_out, dtype=torch.float32, device="cuda")
        t_ws = torch.empty(plan.ws_bytes, dtype=torch.uint8, device="cuda")
        us_topk = timed_events(lambda: ks.grad_topk_select(g_dev, plan, out_idx=t_idx, out_val=t_val, ws=t_ws), 20)
        bytes_topk = g_host.size * 4.0 + plan.n_out * 8.0  # algorithmic: every gradient read once, the selection written
        grad_topk = dict(problem=f"{len(sizes)} tensors, {g_host.size} gradients, k = 0.1 % per tensor ({plan.n_out} selected), "
                                 f"{plan.n_workgroups} steps in {plan.n_launches} launches ({plan.n_filtered_chunks} of them chunks filtered by a sampled "
                                 f"threshold; at most {max(plan.chunks())} chunks per tensor)",
                         us_per_call=round(us_topk, 1), gradients_per_s=round(g_host.size / (us_topk * 1e-6), 1))
        grad_topk.update(hbm_entry(us_topk, bytes_topk))
        if not args.no_cpu_baseline:
            import oracle as orc_t
            t = time.perf_counter()
            e_idx, e_val = orc_t.topk_group(g_host, offs, kk)
            t_orc = time.perf_counter() - t
            grad_topk["cpu_oracle_s"] = round(t_orc, 2)
            grad_topk["cpu_oracle_cores"] = orc_t.num_threads()
            if not args.no_parity:
                grad_topk["exact"] = bool(np.array_equal(t_idx.cpu().numpy(), e_idx)
                                          and np.array_equal(t_val.cpu().numpy().view(np.uint32), e_val.view(np.uint32)))
        log(f"[bench] top-k selection of a ResNet-50 gradient set: {grad_topk}")
        del g_dev

    # ---- CPU oracle on the same inputs: baseline + full-size parity of the first step -----------------------
    cpu_baseline, parity = None, None
    if not args.no_cpu_baseline:
        import oracle as orc
        threads = orc.num_threads()
        G_orc, rows, lists, t_graph = oracle_graph_for_labels(orc, W, y, cfg)
        t_steps = []
        for _ in range(3):                      # best of three
            t = time.perf_counter()
            active, A_orc, tpos = orc.select_active(y, G_orc, C, M)
            ref = orc.knn_softmax_fwd_bwd(W, X, active[:A_orc], tpos, scale, grad_scale)
            ref_dW32 = ref["dWA"].astype(np.float32)
            orc.apply_weight_grad(W, active[:A_orc], ref_dW32, alpha, want_bf16=False)
            t_steps.append(time.perf_counter() - t)
        t_step = min(t_steps)
        cpu_baseline = dict(value=round(B / t_step, 2), unit="samples/s", cores=threads, kind="oracle",
                            sample=f"one whole step (select + fwd/bwd + weight update) on the same batch, A={A_orc}, best of 3; "
                                   f"its graph rows by brute force on the {len(rows)} distinct labels",
                            graph_rows_per_s=round(len(rows) / t_graph, 2),
                            graph_build_s_scaled_to_C=round(t_graph / len(rows) * C, 1))
        log(f"[bench] oracle: step {t_step:.2f}s (best of {[round(v, 2) for v in t_steps]}) on {threads} threads; "
            f"graph rows {len(rows)} in {t_graph:.2f}s")
        if not args.no_parity:
            sys.path.insert(0, os.path.join(ROOT, "tests"))
            from gradcheck import grad_floors, row_errors   # the per-row bound of the parity tests (no oracle code in it)
            g_rows = graph[torch.from_numpy(rows.astype(np.int64)).cuda()].cpu().numpy()
            f_dx, f_dw = grad_floors(W[active[:A_orc]], X, tpos, ref["lse"], scale, grad_scale / B)
            rx = row_errors(first["dX"].cpu().numpy(), ref["dX"], f_dx)
            rw = row_errors(first["dW_active"].cpu().numpy(), ref["dWA"], f_dw) if A == A_orc else None
            parity = dict(
                graph_rows_checked=int(len(rows)), graph_rows_exact=bool((g_rows == lists).all()),
                active_exact=bool(A == A_orc and (first["active_idx"].cpu().numpy() == active).all()
                                  and (first["target_pos"].cpu().numpy() == tpos).all()),
                loss_rel_err=abs(float(first["loss_mean"].item()) - ref["loss"]) / abs(ref["loss"]),
                dX=dict(rows=B, rows_beyond_allowance=rx["n_bad"], worst_row_share_of_allowance=round(rx["worst_ratio"], 3),
                        rel_fro=rx["rel_fro"], max_abs=rx["max_abs"]),
                dW=None if rw is None else dict(rows=A, rows_beyond_allowance=rw["n_bad"],
                                                worst_row_share_of_allowance=round(rw["worst_ratio"], 3), rel_fro=rw["rel_fro"],
                                                max_abs=rw["max_abs"]),
                bound="per row: |got - ref| <= 2e-2 |ref| + floor from the bf16 storage of the logit gradient (tests/gradcheck.py)")
            log(f"[bench] parity of the first step vs the oracle: {parity}")

    # ---- the 1M-class workload: KNN step next to the full softmax over all classes (the paper's Table 3 contrast) ----
    dense_contrast = None
    if args.workload == "shard390k" and not args.headline_only:
        del run, out, ws, first, W_bf, W_master, graph, W
        torch.cuda.empty_cache()
        cfg_d = dict(synth.CONFIGS["dense1m"])
        Cd, Dd, Bd, Kd, Md = cfg_d["C"], cfg_d["D"], cfg_d["B"], cfg_d["K"], cfg_d["M"]
        Wd, Xd, yd = make_inputs(cfg_d)
        graph_d = torch.from_numpy(arithmetic_graph(Cd, Kd)).cuda()   # the step does not depend on the lists being true neighbours
        run_d = StepRunner(ks, torch, hev, cfg_d, Wd, Xd, yd, graph_d, True, True)
        n_d = max(5, args.steps // 5)
        ms_knn, ms_knn_med, _ = run_d.run(n_d, 2, with_stages=False)
        A_d = run_d.A
        f_ws = torch.empty(ks.full_softmax_workspace(Cd, Dd, Bd), dtype=torch.uint8, device="cuda")
        f_out = ks.full_softmax_fwd_bwd(run_d.W_bf, run_d.X_bf, run_d.labels, cfg_d["scale"], 128.0, ws=f_ws, unit_rows=True)
        us_full = timed_events(lambda: ks.full_softmax_fwd_bwd(run_d.W_bf, run_d.X_bf, run_d.labels, cfg_d["scale"], 128.0, out=f_out,
                                                              ws=f_ws, unit_rows=True), max(3, n_d // 2), warm=1)
        assert int(f_out["dev_status"].item()) == 0
        fl_knn, fl_full = 6.0 * Bd * A_d * Dd, 6.0 * Bd * Cd * Dd
        dense_contrast = dict(workload=f"dense1m: C={Cd} D={Dd} B={Bd} K={Kd} M={Md} labels=uniform, lists by an arithmetic pattern",
                              knn_step=dict(active_classes=A_d, ms_per_step=round(ms_knn, 4), samples_per_s=round(Bd / (ms_knn * 1e-3), 1),
                                            what="select + fwd/bwd + weight update", tflops=round(fl_knn / (ms_knn * 1e-3) / 1e12, 1),
                                            frac=round(fl_knn / (ms_knn * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)),
                              full_softmax=dict(ms_per_step=round(us_full * 1e-3, 4), samples_per_s=round(Bd / (us_full * 1e-6), 1),
                                                what="fwd/bwd over all classes, dense dW stored (no update)",
                                                tflops=round(fl_full / (us_full * 1e-6) / 1e12, 1),
                                                frac=round(fl_full / (us_full * 1e-6) / 1e12 / PEAK_BF16_TFLOPS, 4)),
                              knn_speedup=round(us_full * 1e-3 / ms_knn, 2))
        # the graph of this workload (K = 64, k' = 128), built for its time only
        del f_ws, f_out
        gd_ws = torch.empty(ks.knn_graph_build_workspace(Cd, Dd, Kd, 0), dtype=torch.uint8, device="cuda")
        gd_ms = []
        for _ in range(2):
            hev.record(gev[0], stream)
            ks.knn_graph_build(run_d.W_bf, Kd, graph=graph_d, ws=gd_ws)
            hev.record(gev[1], stream)
            torch.cuda.synchronize()
            gd_ms.append(hev.elapsed_ms(gev[0], gev[1]))
        del gd_ws
        gd_tflops = 2.0 * Cd * Cd * Dd / (min(gd_ms) * 1e-3) / 1e12
        dense_contrast["graph_build"] = dict(ms=round(min(gd_ms), 1), tflops=round(gd_tflops, 1), bound="mfma",
                                             **fracs(gd_tflops, PEAK_BF16_TFLOPS, mfma_peak))
        log(f"[bench] dense1m: KNN step {ms_knn:.3f} ms (A={A_d}) vs full softmax {us_full * 1e-3:.3f} ms; graph build "
            f"{min(gd_ms):.0f} ms ({gd_tflops / PEAK_BF16_TFLOPS:.1%} of bf16 peak)")

    graph_e = {"ms": round(graph_best, 2), "tflops": round(graph_tflops, 1), "bound": "mfma"}
    graph_e.update(fracs(graph_tflops, PEAK_BF16_TFLOPS, mfma_peak))
    n_sym_wg, _ = ks.knn_graph_build_plan(C, D, K, 0)
    if n_sym_wg:
        # the rate above is algorithmic (2 C^2 D flop: every row against every row); the matrix cores execute less
        streamed = 0
        for wg in range(n_sym_wg):
            p12 = ks.knn_graph_build_plan(C, D, K, 0, wg)[1]
            if p12[0] >= 0:
                streamed += sum(max(0, p12[2 + 2 * q] - p12[1 + 2 * q]) for q in range(5))
        graph_e["flops_executed_over_algorithmic"] = round(streamed * 256 / (C * C) + 1.0 / 32, 4)
        graph_e["note"] = ("similarities are symmetric: every pair of rows is multiplied once and used for both rows, after a "
                           "pass over every 32nd row that fixes the rows' thresholds")
    res = {
        "metric": "KNN-softmax fwd+bwd samples/sec per GPU", "value": round(value, 1), "unit": "samples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_hip_event_median": round(ms_median, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: C={C} D={D} B={B} K={K} M={M} labels={cfg['labels']} s={scale}",
                   "active_classes": A,
                   "step": ("knn_softmax_fwd_bwd_update_selected_next, one call per step: fwd/bwd + weight update of batch n and "
                            "the selection (Algorithm 1) of batch n + 1 in the same launches, the list read in place from the "
                            "buffers the previous call wrote (KS_FLAG_TRUSTED_LIST); the one-call step that selects "
                            "its own batch first is selection_variants.serial_ms_per_step") if next_inside
                   else ("knn_softmax_fwd_bwd_update (select + fwd/bwd + weight update in one call)" if fused_update
                         else "select + knn_softmax_fwd_bwd + apply_weight_grad"),
                   "unit_rows_flag": unit_rows},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "measured_peaks": peaks,
        "whole_step": whole_step,
        "phases": phases,
        "graph_build": graph_e,
        "selection_variants": selection_variants,
        "at_the_cap": at_the_cap,
        "dense_contrast": dense_contrast,
        "gather_rows": gather,
        "normalized_layer": normalized_layer,
        "sharded_node": sharded_node,
        "grad_topk": grad_topk,
        "parity": parity,
    }
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
