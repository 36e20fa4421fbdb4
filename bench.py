#!/usr/bin/env python3
"""Benchmark of the KNN-softmax hot path on one MI355X.

A "step" is one pass of the whole path over one synthetic batch: active-class selection, logits GEMM
(with the row gather), softmax / cross-entropy / logit gradient, dX and dW GEMMs, and the weight update
(knn_softmax_fwd_bwd + apply_weight_grad).  The KNN graph is rebuilt once before the loop
(knn_graph_build, the once-per-epoch stage) and timed separately.

Prints ONE JSON line on stdout: whole-job samples/s, the roofline figure of the dominant kernel (from
HIP events recorded around every stage inside the timed region) and the CPU oracle timed on the host
cores on the same inputs.  Everything else goes to stderr.
"""
from __future__ import annotations

import argparse
import ctypes as ct
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

PHASES = ["select", "logits_gemm", "row_stats", "logit_grad", "dx_gemm", "dx_reduce", "dw_gemm", "apply"]

# HBM bytes per launch of each stage's kernel from two rocprofv3 --pmc runs (FETCH_SIZE scaled by 2.0, WRITE_SIZE by
# 1.0, the factors a copy of known size gives), copied from profiles/bench_shard390k_hbm_traffic.txt
# (unit-rows mode: one softmax sweep; the dW launch also carries the reduction of the dX partial sums)
MEASURED_TRAFFIC = {
    ("shard390k", "logits_gemm"): 62.56e6,
    ("shard390k", "dx_gemm"): 87.42e6,
    ("shard390k", "dw_gemm"): 169.40e6,          # with the weight update inside the kernel (the default step)
    ("shard390k", "dw_gemm_separate"): 117.78e6,  # --separate-update
    ("shard390k", "apply"): 125.50e6,
}


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

    def destroy(self, evs):
        for e in evs:
            self.hip.hipEventDestroy(ct.c_void_p(e))


def make_inputs(cfg, log_fn=log):
    import synth
    t = time.time()
    W, X = synth.make_WX(cfg)
    y = synth.make_labels(cfg)
    log_fn(f"[bench] inputs: C={cfg['C']} D={cfg['D']} B={cfg['B']} K={cfg['K']} M={cfg['M']} labels={cfg['labels']} "
           f"({time.time() - t:.1f}s host generation)")
    return W, X, y


def oracle_graph_for_labels(orc, W, y, cfg):
    """Neighbour lists for the oracle: exact brute force for the rows the selection reads (the labels), a
    synthetic filler elsewhere (never read).  Returns (G, distinct rows, their lists, seconds)."""
    import synth
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
    B, D, K, C = cfg["B"], cfg["D"], cfg["K"], cfg["C"]
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="shard390k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-parity", action="store_true")
    ap.add_argument("--headline-only", action="store_true",
                    help="only the headline step (no normalised-layer and sharded-node measurements): used for the profiles")
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
    grad_scale, lr = 128.0, 0.05
    alpha = -lr / grad_scale

    W, X, y = make_inputs(cfg)
    W_bf = torch.from_numpy(W).cuda().to(torch.bfloat16)
    W_master = torch.from_numpy(W).cuda()
    X_bf = torch.from_numpy(X).cuda().to(torch.bfloat16)
    labels = torch.from_numpy(y).cuda()
    stream = torch.cuda.current_stream().cuda_stream
    hev = HipEvents()

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

    # ---- step buffers -----------------------------------------------------------------------------------
    ws = torch.empty(ks.knn_softmax_workspace(C, D, B, K, M), dtype=torch.uint8, device="cuda")
    # the synthetic rows are L2-normalised, as the paper's are: the library may rely on it
    unit_rows = not args.general_rows
    fused_update = not args.separate_update
    out = ks.knn_softmax_fwd_bwd(W_bf, X_bf, labels, graph, M, scale, grad_scale, ws=ws, unit_rows=unit_rows)
    torch.cuda.synchronize()
    A = int(out["n_active"].item())
    assert int(out["dev_status"].item()) == 0
    log(f"[bench] active classes A={A} of M={M}")
    first = {k: out[k].clone() for k in ("active_idx", "target_pos", "loss_per_sample", "loss_mean", "dX")}
    first["dW_active"] = out["dW_active"][:A].clone()

    out_fused = dict(out)
    out_fused["dW_active"] = None      # the fused step does not store the gradient rows
    L = ks.lib()
    n_ev = 9
    evs = [hev.create(n_ev) for _ in range(args.steps)]

    def step(ev=None):
        if ev is None and fused_update:
            ks.knn_softmax_fwd_bwd_update(W_master, W_bf, X_bf, labels, graph, M, scale, grad_scale, alpha, out=out_fused,
                                          ws=ws, unit_rows=unit_rows)
            return
        if ev is None:
            ks.knn_softmax_fwd_bwd(W_bf, X_bf, labels, graph, M, scale, grad_scale, out=out, ws=ws,
                                   unit_rows=unit_rows)
        else:
            rc = L.knn_softmax_fwd_bwd_profiled(
                ct.c_void_p(W_master.data_ptr() if fused_update else 0), ct.c_void_p(W_bf.data_ptr()),
                ct.c_void_p(X_bf.data_ptr()), ct.c_void_p(labels.data_ptr()),
                ct.c_void_p(graph.data_ptr()), ct.c_int64(C), ct.c_int(D), ct.c_int(B), ct.c_int(K), ct.c_int(M),
                ct.c_float(scale), ct.c_float(grad_scale), ct.c_float(alpha), ct.c_uint32(1 if unit_rows else 0),
                ct.c_void_p(out["active_idx"].data_ptr()),
                ct.c_void_p(out["n_active"].data_ptr()), ct.c_void_p(out["target_pos"].data_ptr()),
                ct.c_void_p(out["loss_per_sample"].data_ptr()), ct.c_void_p(out["loss_mean"].data_ptr()),
                ct.c_void_p(out["dX"].data_ptr()), ct.c_void_p(0 if fused_update else out["dW_active"].data_ptr()),
                ct.c_void_p(ws.data_ptr()), ct.c_size_t(ws.numel()), ct.c_void_p(out["dev_status"].data_ptr()),
                ct.c_void_p(stream), ev, ct.c_int(8))
            assert rc == 0, rc
        if not fused_update:
            ks.apply_weight_grad(W_master, W_bf, out["active_idx"], out["n_active"], out["dW_active"], alpha,
                                 idx_sorted_unique=True, ws=ws, dev_status=out["dev_status"])
        if ev is not None:
            hev.record(ev[8], stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # timed region: K steps, nothing but the library's own launches on the stream
    t0 = time.perf_counter()
    for s in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = B / (ms_per_step * 1e-3)
    assert int(out["dev_status"].item()) == 0
    # the same K steps again with a HIP event recorded at every stage boundary (the event records cost a
    # few microseconds each, which is why they are kept out of the region that `value` is measured on)
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(evs[s])
    torch.cuda.synchronize()
    ms_per_step_instrumented = (time.perf_counter() - t0) * 1e3 / args.steps
    assert int(out["dev_status"].item()) == 0

    # per-stage durations from the events of the timed region
    dur = {p: 0.0 for p in PHASES}
    for ev in evs:
        for k, p in enumerate(PHASES):
            dur[p] += hev.elapsed_ms(ev[k], ev[k + 1])
    for p in PHASES:
        dur[p] = dur[p] / args.steps * 1e3  # microseconds
    model = phase_model(cfg, A, unit_rows, fused_update)
    phases = {}
    for p in PHASES:
        m = model[p]
        e = dict(us=round(dur[p], 2), bound=m["bound"])
        if "flops" in m:
            e["tflops"] = round(m["flops"] / (dur[p] * 1e-6) / 1e12, 1)
            e["frac"] = round(e["tflops"] / PEAK_BF16_TFLOPS, 4)
        elif "bytes" in m:
            e["gbs"] = round(m["bytes"] / (dur[p] * 1e-6) / 1e9, 1)
            e["frac"] = round(e["gbs"] / PEAK_HBM_GBS, 4)
        phases[p] = e
    log("[bench] stage times (us): " + ", ".join(f"{p}={phases[p]['us']}" for p in PHASES))
    dom = max((p for p in PHASES if model[p]["bound"] in ("mfma", "hbm")), key=lambda p: dur[p])
    key = "dw_gemm_separate" if (dom == "dw_gemm" and not fused_update) else dom
    traffic = MEASURED_TRAFFIC.get((args.workload, key)) if unit_rows else None  # measured in unit-rows mode only
    if model[dom]["bound"] == "mfma":
        roofline = dict(bound="mfma", achieved=phases[dom]["tflops"], peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                        frac=phases[dom]["frac"], traffic=traffic, kernel=dom)
        if dom == "dw_gemm" and fused_update:
            # this launch is two things: the dW contraction (the flops counted above) and the weight update of the
            # active rows in its epilogue, which is HBM work; both against their own peaks, one after the other
            upd_bytes = A * D * (4.0 + 4.0 + 2.0)
            t_roof = model[dom]["flops"] / (PEAK_BF16_TFLOPS * 1e12) + upd_bytes / (PEAK_HBM_GBS * 1e9)
            roofline.update(kernel="dw_gemm + weight update (one launch)", update_bytes=upd_bytes,
                            frac_of_two_phase_roofline=round(t_roof / (dur[dom] * 1e-6), 4),
                            runner_up=dict(kernel="logits_gemm", bound="mfma", achieved=phases["logits_gemm"]["tflops"],
                                           frac=phases["logits_gemm"]["frac"], us=phases["logits_gemm"]["us"],
                                           traffic=MEASURED_TRAFFIC.get((args.workload, "logits_gemm")) if unit_rows else None))
    else:
        roofline = dict(bound="hbm", achieved=phases[dom]["gbs"], peak=PEAK_HBM_GBS, unit="GB/s",
                        frac=phases[dom]["frac"], traffic=traffic, kernel=dom)

    # ---- the row gather as a kernel of its own (in the step it is fused into the loaders of the contractions):
    # A rows of D bf16 values read and written once
    gather = None
    if not args.headline_only:
        gev = hev.create(2)
        g_out = torch.empty((M, D), dtype=torch.bfloat16, device="cuda")
        g_st = torch.zeros(1, dtype=torch.int32, device="cuda")
        for _ in range(3):
            ks.knn_gather_rows(W_bf, out["active_idx"], out["n_active"], out=g_out, dev_status=g_st)
        hev.record(gev[0], stream)
        for _ in range(20):
            ks.knn_gather_rows(W_bf, out["active_idx"], out["n_active"], out=g_out, dev_status=g_st)
        hev.record(gev[1], stream)
        torch.cuda.synchronize()
        us_g = hev.elapsed_ms(gev[0], gev[1]) * 1e3 / 20
        bytes_g = A * D * 2.0 * 2
        gather = dict(us=round(us_g, 2), bound="hbm", gbs=round(bytes_g / (us_g * 1e-6) / 1e9, 1),
                      frac=round(bytes_g / (us_g * 1e-6) / 1e9 / PEAK_HBM_GBS, 4))
        log(f"[bench] stand-alone gather of the {A} active rows: {gather}")

    normalized_layer = None
    nev = hev.create(2)
    if not args.headline_only:
        # ---- the layer with un-normalised fp32 weights (normalisation inside the layer, Section 3.2.1): the same step
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
        hev.record(nev[0], stream)
        for s in range(args.steps):
            ks.apply_weight_grad_normalized(W_master, W_bf, inv_norm, out["active_idx"], out["n_active"], out["dW_active"],
                                            alpha, idx_sorted_unique=True, ws=ws, dev_status=out["dev_status"])
        hev.record(nev[1], stream)
        torch.cuda.synchronize()
        us_apply_n = hev.elapsed_ms(nev[0], nev[1]) * 1e3 / args.steps
        assert int(out["dev_status"].item()) == 0
        bytes_apply_n = A * (D * (4.0 + 4.0 + 4.0 + 2.0) + 4.0)
        normalized_layer = dict(ms_per_step=round(ms_norm_step, 4), samples_per_s=round(B / (ms_norm_step * 1e-3), 1),
                                step="normalize X + select + knn_softmax_fwd_bwd + project dX + apply_weight_grad_normalized",
                                apply_normalized=dict(us=round(us_apply_n, 2), bound="hbm",
                                                      gbs=round(bytes_apply_n / (us_apply_n * 1e-6) / 1e9, 1),
                                                      frac=round(bytes_apply_n / (us_apply_n * 1e-6) / 1e9 / PEAK_HBM_GBS, 4)))
        log(f"[bench] layer with normalisation inside: {ms_norm_step:.4f} ms/step, apply_normalized {us_apply_n:.1f} us")

    # ---- this GPU as one node of four (Section 3.2.3): graph compression and selection on the compressed graph,
    # with and without the random fill-up to M (Algorithm 1); integer work, bit-exact against the oracle in the tests
    sharded_node = None
    if args.workload == "shard390k" and not args.headline_only:
        Cg4, c0 = 4 * C, C
        cc = np.arange(Cg4, dtype=np.int64)[:, None]
        kk = np.arange(K, dtype=np.int64)[None, :]
        G4 = torch.from_numpy(((cc + 1 + (cc * 2654435761 + kk * 40503) % (Cg4 - 1)) % Cg4).astype(np.int32)).cuda()
        y4 = torch.from_numpy(synth.labels_zipf(cfg["seed"], B, Cg4, 1.1)).cuda()
        counts, offsets, flat, st4 = ks.knn_graph_compress(G4, c0, C)
        c_ws = torch.empty(int(L.knn_graph_compress_workspace(ct.c_int64(Cg4), ct.c_int(K))), dtype=torch.uint8, device="cuda")
        s_ws = torch.empty(ks.knn_select_active_csr_workspace(C, B, K, M), dtype=torch.uint8, device="cuda")

        def timed(fn, reps):
            fn()
            hev.record(nev[0], stream)
            for _ in range(reps):
                fn()
            hev.record(nev[1], stream)
            torch.cuda.synchronize()
            return hev.elapsed_ms(nev[0], nev[1]) * 1e3 / reps

        def compress():
            rc = L.knn_graph_compress(ct.c_void_p(G4.data_ptr()), ct.c_int64(Cg4), ct.c_int(K), ct.c_int64(c0), ct.c_int64(C),
                                      ct.c_void_p(counts.data_ptr()), ct.c_void_p(offsets.data_ptr()),
                                      ct.c_void_p(flat.data_ptr()), ct.c_int64(flat.numel()), ct.c_void_p(c_ws.data_ptr()),
                                      ct.c_size_t(c_ws.numel()), ct.c_void_p(st4.data_ptr()), ct.c_void_p(stream))
            assert rc == 0, rc

        us_compress = timed(compress, 10)
        us_sel = timed(lambda: ks.knn_select_active_csr(y4, counts, offsets, flat, c0, C, K, M, ws=s_ws, dev_status=st4), 20)
        us_sel_pad = timed(lambda: ks.knn_select_active_csr(y4, counts, offsets, flat, c0, C, K, M, pad_random=True, pad_seed=1,
                                                            ws=s_ws, dev_status=st4), 20)
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
        n_act4 = int(node_step(False)["n_active"].item())
        torch.cuda.synchronize()
        assert int(st4.item()) == 0
        bytes_c = Cg4 * K * 4.0 * 2 + flat.numel() * 4.0 + Cg4 * (4.0 * 2 + 8.0)
        sharded_node = dict(problem=f"Cg={Cg4} classes on 4 nodes, this node owns [{c0}, {c0 + C}); K={K}, global batch {B}",
                            compressed_entries=int(flat.numel()), classes_found=int(o4["n_found"].item()),
                            graph_compress=dict(us=round(us_compress, 1), bound="hbm",
                                                gbs=round(bytes_c / (us_compress * 1e-6) / 1e9, 1),
                                                frac=round(bytes_c / (us_compress * 1e-6) / 1e9 / PEAK_HBM_GBS, 4)),
                            select_csr_us=round(us_sel, 2), select_csr_with_fill_up_us=round(us_sel_pad, 2),
                            node_step=dict(what="select_csr + fwd_stats + exchange stand-in + bwd_from_stats + "
                                                "apply_weight_grad_normalized, one-sweep softmax",
                                           ms_per_step=round(ms_node, 4), active_classes=n_act4,
                                           ms_per_step_filled_to_M=round(ms_node_pad, 4)))
        log(f"[bench] one node of four: compress {us_compress:.0f} us, select {us_sel:.1f} us, with fill-up {us_sel_pad:.1f} us; "
            f"node step {ms_node:.4f} ms (A={n_act4}), filled to M {ms_node_pad:.4f} ms")
        del G4

    # ---- second workload (Section 3.3.2): layer-wise top-k selection over the gradient set of a ResNet-50, 99.9 %
    # sparsity, all 161 tensors in one call (two launches); HBM-bound: every gradient is read once
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
        tev = hev.create(3)
        reps = 20

        def topk_call():
            ks.grad_topk_select(g_dev, plan, out_idx=t_idx, out_val=t_val, ws=t_ws)

        for _ in range(3):
            topk_call()
        hev.record(tev[0], stream)
        for _ in range(reps):
            topk_call()
        hev.record(tev[1], stream)
        torch.cuda.synchronize()
        us_topk = hev.elapsed_ms(tev[0], tev[1]) * 1e3 / reps
        bytes_topk = g_host.size * 4.0 + plan.n_out * 8.0  # algorithmic: every gradient read once, the selection written
        grad_topk = dict(problem=f"{len(sizes)} tensors, {g_host.size} gradients, k = 0.1 % per tensor ({plan.n_out} selected), "
                                 f"{plan.n_workgroups} selection steps in {plan.n_levels} launches (at most {max(plan.chunks())} chunks per tensor)",
                         us_per_call=round(us_topk, 1), gradients_per_s=round(g_host.size / (us_topk * 1e-6), 1),
                         bound="hbm", gbs=round(bytes_topk / (us_topk * 1e-6) / 1e9, 1),
                         frac=round(bytes_topk / (us_topk * 1e-6) / 1e9 / PEAK_HBM_GBS, 4))
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
        t = time.perf_counter()
        active, A_orc, tpos = orc.select_active(y, G_orc, C, M)
        ref = orc.knn_softmax_fwd_bwd(W, X, active[:A_orc], tpos, scale, grad_scale)
        ref_dW32 = ref["dWA"].astype(np.float32)
        orc.apply_weight_grad(W, active[:A_orc], ref_dW32, alpha, want_bf16=False)
        t_step = time.perf_counter() - t
        cpu_baseline = dict(value=round(B / t_step, 2), unit="samples/s", cores=threads, kind="oracle",
                            sample=f"one whole step (select + fwd/bwd + weight update) on the same batch, A={A_orc}; "
                                   f"its graph rows by brute force on the {len(rows)} distinct labels",
                            graph_rows_per_s=round(len(rows) / t_graph, 2),
                            graph_build_s_scaled_to_C=round(t_graph / len(rows) * C, 1))
        log(f"[bench] oracle: step {t_step:.2f}s on {threads} threads; graph rows {len(rows)} in {t_graph:.2f}s")
        if not args.no_parity:
            g_rows = graph[torch.from_numpy(rows.astype(np.int64)).cuda()].cpu().numpy()

            def relf(a, b):
                return float(np.linalg.norm(a.astype(np.float64) - b) / np.linalg.norm(b))

            parity = dict(
                graph_rows_checked=int(len(rows)), graph_rows_exact=bool((g_rows == lists).all()),
                active_exact=bool(A == A_orc and (first["active_idx"].cpu().numpy() == active).all()
                                  and (first["target_pos"].cpu().numpy() == tpos).all()),
                loss_rel_err=abs(float(first["loss_mean"].item()) - ref["loss"]) / abs(ref["loss"]),
                dX_rel_fro=relf(first["dX"].cpu().numpy(), ref["dX"]),
                dW_rel_fro=relf(first["dW_active"].cpu().numpy(), ref["dWA"]))
            log(f"[bench] parity of the first step vs the oracle: {parity}")

    res = {
        "metric": "KNN-softmax fwd+bwd samples/sec per GPU", "value": round(value, 1), "unit": "samples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_with_stage_events": round(ms_per_step_instrumented, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: C={C} D={D} B={B} K={K} M={M} labels={cfg['labels']} s={scale}",
                   "active_classes": A, "step": "knn_softmax_fwd_bwd_update (select + fwd/bwd + weight update in one call)" if fused_update
                   else "select + knn_softmax_fwd_bwd + apply_weight_grad",
                   "unit_rows_flag": unit_rows},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "phases": phases,
        "graph_build": {"ms": round(graph_best, 2), "tflops": round(graph_tflops, 1),
                        "frac": round(graph_tflops / PEAK_BF16_TFLOPS, 4), "bound": "mfma"},
        "gather_rows": gather,
        "normalized_layer": normalized_layer,
        "sharded_node": sharded_node,
        "grad_topk": grad_topk,
        "parity": parity,
    }
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
