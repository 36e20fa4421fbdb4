"""GPU parity at the full size of the headline workload (C=390,625, D=512, B=1,024, K=32, M=32,768; Zipf and
uniform labels), in the launch configuration the benchmark times.  The oracle cannot brute-force the whole
graph at this size, so the neighbour lists are checked on sampled rows (every distinct label of the batch
plus random rows); selection, loss and gradients of one step are then compared in full, with the oracle
working from its own brute-forced lists for the label rows.  The weight update is compared on every touched
row, and sampled untouched rows must keep their bits."""
import numpy as np
import pytest
import torch

import synth
from gradcheck import check_step_grads

pytestmark = pytest.mark.gpu

LOSS_RTOL = 1e-3
SENTINEL = -12345.0


@pytest.fixture(scope="module")
def ks():
    import paper_2102_06025_amd as ks
    ks.lib()
    assert torch.cuda.is_available(), "these tests need the GPU"
    return ks


@pytest.fixture(scope="module")
def shard(ks):
    """Inputs of the headline shard and the GPU-built graph (shared by the cases below)."""
    cfg = synth.CONFIGS["shard390k"]
    print(f"[case] generating shard390k inputs C={cfg['C']} D={cfg['D']}", flush=True)
    W, X = synth.make_WX(cfg)
    W_bf = torch.from_numpy(W).cuda().to(torch.bfloat16)
    print("[case] knn_graph_build on the full shard", flush=True)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    graph, sims = ks.knn_graph_build(W_bf, cfg["K"], want_sims=True, dev_status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    return dict(cfg=cfg, W=W, X=X, W_bf=W_bf, graph=graph, sims=sims)


def _buffers(B, D, M):
    """Output buffers of a step whose gradient matrices start from a sentinel."""
    return dict(active_idx=torch.empty(M, dtype=torch.int32, device="cuda"),
                n_active=torch.empty(1, dtype=torch.int32, device="cuda"),
                target_pos=torch.empty(B, dtype=torch.int32, device="cuda"),
                loss_per_sample=torch.empty(B, dtype=torch.float32, device="cuda"),
                loss_mean=torch.empty(1, dtype=torch.float32, device="cuda"),
                dX=torch.full((B, D), SENTINEL, dtype=torch.float32, device="cuda"),
                dW_active=torch.full((M, D), SENTINEL, dtype=torch.float32, device="cuda"))


def test_graph_sampled_rows_exact(ks, orc, shard):
    cfg, W = shard["cfg"], shard["W"]
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([rng.integers(0, cfg["C"], 192), [0, cfg["C"] - 1]])).astype(np.int32)
    print(f"[case] graph rows by brute force: {len(rows)} sampled rows", flush=True)
    lists, sims = orc.graph_bruteforce(W, cfg["K"], rows)
    sel = torch.from_numpy(rows.astype(np.int64)).cuda()
    g = shard["graph"][sel].cpu().numpy()
    s = shard["sims"][sel].cpu().numpy()
    assert (g == lists).all()
    assert np.abs(s - sims).max() <= 1e-6
    # properties that hold for every row: no self, ids in range, distinct, similarities non-increasing
    G = shard["graph"]
    ar = torch.arange(cfg["C"], device="cuda", dtype=torch.int32)[:, None]
    assert bool(((G >= 0) & (G < cfg["C"]) & (G != ar)).all())
    srt = torch.sort(G, dim=1).values
    assert bool((srt[:, 1:] != srt[:, :-1]).all())
    S = shard["sims"]
    assert bool((S[:, 1:] <= S[:, :-1]).all())


@pytest.mark.parametrize("K", [32, 64])
def test_graph_of_clustered_rows_sampled_rows_exact(ks, orc, K):
    """The headline shard with clustered class weights (neighbour lists overlap heavily, some rows are in the lists of
    hundreds of others): the graph build that computes every similarity once must neither lose a neighbour nor send
    rows to its exhaustive pass in numbers that would show in the time -- with the shard's K = 32 (k' = 48) and with
    K = 64 (k' = 128)."""
    cfg = synth.CONFIGS["shard390k_clustered"]
    print(f"[case] generating clustered rows C={cfg['C']} D={cfg['D']}, K={K}", flush=True)
    W, _ = synth.make_WX(cfg)
    W_bf = torch.from_numpy(W).cuda().to(torch.bfloat16)
    graph, sims = ks.knn_graph_build(W_bf, K, want_sims=True)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    ks.knn_graph_build(W_bf, K, graph=graph, sims=sims)
    e1.record()
    torch.cuda.synchronize()
    print(f"[case] clustered graph build {e0.elapsed_time(e1):.1f} ms", flush=True)
    assert e0.elapsed_time(e1) < 400.0   # (≈ 100 ms; a row in the exhaustive pass costs about a millisecond)
    rng = np.random.default_rng(11)
    rows = np.unique(np.concatenate([rng.integers(0, cfg["C"], 62), [0, cfg["C"] - 1]])).astype(np.int32)
    print(f"[case] graph rows by brute force: {len(rows)} sampled rows", flush=True)
    lists, ref = orc.graph_bruteforce(W, K, rows)
    sel = torch.from_numpy(rows.astype(np.int64)).cuda()
    assert (graph[sel].cpu().numpy() == lists).all()
    assert np.abs(sims[sel].cpu().numpy() - ref).max() <= 1e-6


@pytest.mark.parametrize("name,unit_rows", [("shard390k", True), ("shard390k", False), ("shard390k_uniform", True)])
def test_step_full_size(ks, orc, shard, name, unit_rows):
    cfg = synth.CONFIGS[name]
    C, D, B, K, M, scale = cfg["C"], cfg["D"], cfg["B"], cfg["K"], cfg["M"], cfg["scale"]
    W, X, W_bf, graph = shard["W"], shard["X"], shard["W_bf"], shard["graph"]
    y = synth.make_labels(cfg)
    grad_scale, alpha = 128.0, -0.05 / 128.0
    print(f"[case] {name}: fwd_bwd + apply at full size, B={B} M={M} unit_rows={unit_rows}", flush=True)
    X_bf = torch.from_numpy(X).cuda().to(torch.bfloat16)
    out = ks.knn_softmax_fwd_bwd(W_bf, X_bf, torch.from_numpy(y).cuda(), graph, M, scale, grad_scale, out=_buffers(B, D, M),
                                 unit_rows=unit_rows)
    torch.cuda.synchronize()
    assert int(out["dev_status"].item()) == 0
    A = int(out["n_active"].item())

    # oracle: its own lists for the rows that selection reads
    rows = np.unique(y).astype(np.int32)
    print(f"        oracle: brute-force lists of the {len(rows)} distinct labels", flush=True)
    lists, _ = orc.graph_bruteforce(W, K, rows)
    g_rows = graph[torch.from_numpy(rows.astype(np.int64)).cuda()].cpu().numpy()
    assert (g_rows == lists).all()
    G = np.empty((C, K), dtype=np.int32)
    G[:] = (np.arange(C, dtype=np.int64)[:, None] + 1 + np.arange(K)[None, :]) % C  # never read
    G[rows] = lists
    active, A_ref, tpos = orc.select_active(y, G, C, M)
    assert A == A_ref
    assert (out["active_idx"].cpu().numpy() == active).all()
    assert (out["target_pos"].cpu().numpy() == tpos).all()
    print(f"        oracle: fwd/bwd with A={A_ref}", flush=True)
    ref = orc.knn_softmax_fwd_bwd(W, X, active[:A_ref], tpos, scale, grad_scale)
    li = out["loss_per_sample"].cpu().numpy()
    assert np.abs(li - ref["loss_i"]).max() <= LOSS_RTOL * max(1.0, np.abs(ref["loss_i"]).max())
    loss = float(out["loss_mean"].item())
    assert abs(loss - ref["loss"]) <= LOSS_RTOL * abs(ref["loss"])
    print(f"        A={A} loss={loss:.6f} ref={ref['loss']:.6f}", flush=True)
    # every one of the B rows of dX and of the A rows of dW_A
    check_step_grads(out["dX"].cpu().numpy(), out["dW_active"][:A].cpu().numpy(), ref, W[active[:A]], X, tpos, scale,
                     grad_scale, tag=name)
    assert bool((out["dW_active"][A:] == SENTINEL).all()), "rows beyond n_active were written"

    # weight update with the GPU's own gradient rows (so that only the update arithmetic is compared)
    W_master = torch.from_numpy(W).cuda()
    W_copy = W_bf.clone()
    st = ks.apply_weight_grad(W_master, W_copy, out["active_idx"], out["n_active"], out["dW_active"], alpha,
                              idx_sorted_unique=True)
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    dW32 = out["dW_active"][:A].cpu().numpy()
    W_ref, W_ref_bf = orc.apply_weight_grad(W, active[:A], dW32, alpha, want_bf16=True)
    idx = torch.from_numpy(active[:A].astype(np.int64)).cuda()
    got = W_master[idx].cpu().numpy()
    # one fp32 fused multiply-add per element against the oracle's fp64 sum rounded once: half an ulp each
    assert np.abs(got - W_ref[active[:A]]).max() <= 2.0 ** -23 * np.abs(W_ref[active[:A]]).max()
    got_bf = W_copy[idx].view(torch.int16).cpu().numpy().view(np.uint16)
    # the bf16 copy is the rounding of the GPU's own fp32 master; it equals the oracle's wherever the two
    # masters round the same way
    assert (got_bf == synth.bf16_bits(got)).all()
    assert np.mean(got_bf == W_ref_bf[active[:A]]) > 0.999
    # the whole step in one call (update inside the dW kernel) gives the same bits
    W_master2 = torch.from_numpy(W).cuda()
    W_copy2 = W_bf.clone()
    out2 = ks.knn_softmax_fwd_bwd_update(W_master2, W_copy2, X_bf, torch.from_numpy(y).cuda(), graph, M, scale, grad_scale,
                                         alpha, unit_rows=unit_rows)
    torch.cuda.synchronize()
    assert int(out2["dev_status"].item()) == 0 and out2["dW_active"] is None
    assert torch.equal(out2["dX"], out["dX"]) and torch.equal(out2["loss_mean"], out["loss_mean"])
    assert torch.equal(W_master2, W_master) and torch.equal(W_copy2, W_copy)
    del W_master2, W_copy2, out2
    rng = np.random.default_rng(9)
    untouched = np.setdiff1d(rng.integers(0, C, 4096), active[:A])
    ui = torch.from_numpy(untouched.astype(np.int64)).cuda()
    assert (W_master[ui].cpu().numpy() == W[untouched]).all()
    assert bool((W_copy[ui] == W_bf[ui]).all())


def test_step_dense1m(ks, orc):
    """The largest workload (C = 1,000,000, B = 2,048, K = 64, M = 131,072; about 124,500 active rows): eight
    sample blocks per slab instead of four, and slabs too long for the sweeps' LDS copy of the gather list.
    The neighbour lists are an arithmetic pattern here (what the selection and the softmax do with them does
    not depend on their being true neighbours); both softmax modes against one oracle run."""
    cfg = synth.CONFIGS["dense1m"]
    C, D, B, K, M, scale = cfg["C"], cfg["D"], cfg["B"], cfg["K"], cfg["M"], cfg["scale"]
    print(f"[case] dense1m: generating inputs C={C} D={D} B={B} K={K} M={M}", flush=True)
    W, X = synth.make_WX(cfg)
    y = synth.make_labels(cfg)
    c = np.arange(C, dtype=np.int64)[:, None]
    k = np.arange(K, dtype=np.int64)[None, :]
    G = ((c + 1 + (c * 2654435761 + k * 40503) % (C - 1)) % C).astype(np.int32)  # K distinct ids, none equal to c
    assert (G != c).all() and (np.sort(G[:1000], axis=1)[:, 1:] != np.sort(G[:1000], axis=1)[:, :-1]).all()
    grad_scale = 128.0
    active, A_ref, tpos = orc.select_active(y, G, C, M)
    print(f"        oracle: fwd/bwd with A={A_ref}", flush=True)
    ref = orc.knn_softmax_fwd_bwd(W, X, active[:A_ref], tpos, scale, grad_scale)
    W_bf = torch.from_numpy(W).cuda().to(torch.bfloat16)
    X_bf = torch.from_numpy(X).cuda().to(torch.bfloat16)
    Gd = torch.from_numpy(G).cuda()
    yd = torch.from_numpy(y).cuda()
    for unit_rows in (True, False):
        print(f"[case] dense1m: fwd_bwd unit_rows={unit_rows}", flush=True)
        out = ks.knn_softmax_fwd_bwd(W_bf, X_bf, yd, Gd, M, scale, grad_scale, out=_buffers(B, D, M), unit_rows=unit_rows)
        torch.cuda.synchronize()
        assert int(out["dev_status"].item()) == 0
        assert int(out["n_active"].item()) == A_ref
        assert (out["active_idx"].cpu().numpy() == active).all()
        assert (out["target_pos"].cpu().numpy() == tpos).all()
        li = out["loss_per_sample"].cpu().numpy()
        assert np.abs(li - ref["loss_i"]).max() <= LOSS_RTOL * max(1.0, np.abs(ref["loss_i"]).max())
        loss = float(out["loss_mean"].item())
        assert abs(loss - ref["loss"]) <= LOSS_RTOL * abs(ref["loss"])
        print(f"        A={A_ref} loss={loss:.6f} ref={ref['loss']:.6f}", flush=True)
        check_step_grads(out["dX"].cpu().numpy(), out["dW_active"][:A_ref].cpu().numpy(), ref, W[active[:A_ref]], X, tpos,
                         scale, grad_scale, tag=f"dense1m unit_rows={unit_rows}")
        assert bool((out["dW_active"][A_ref:] == SENTINEL).all()), "rows beyond n_active were written"
        del out


@pytest.mark.parametrize("name", ["shard390k", "shard390k_uniform"])
def test_headline_loop_full_size_equals_the_one_call_step(ks, shard, name):
    """The loop `bench.py` times -- one knn_softmax_fwd_bwd_update_selected_next call per step, the list read in place
    (KS_FLAG_TRUSTED_LIST), the next batch's selection inside the step's launches -- against one-call steps on the same
    three batches (those are the calls the oracle checks above): lists, losses, dX of every step and the weights at the
    end, bit for bit, at the headline size (Zipf labels: 182 dW tiles beside the 32 selection workgroups; uniform
    labels: the cap, 512 tiles)."""
    cfg = synth.CONFIGS[name]
    C, D, B, K, M, scale = cfg["C"], cfg["D"], cfg["B"], cfg["K"], cfg["M"], cfg["scale"]
    W_bf, graph = shard["W_bf"], shard["graph"]
    X_bf = torch.from_numpy(shard["X"]).cuda().to(torch.bfloat16)
    gs, alpha = 128.0, -0.05 / 128.0
    ys = [torch.from_numpy(synth.make_labels(cfg, seed=cfg["seed"] + 31 * t)).cuda() for t in range(4)]
    Wm1, Wb1 = W_bf.float(), W_bf.clone()
    ref = []
    for t in range(3):
        a = ks.knn_softmax_fwd_bwd_update(Wm1, Wb1, X_bf, ys[t], graph, M, scale, gs, alpha, unit_rows=True)
        torch.cuda.synchronize()
        assert int(a["dev_status"].item()) == 0
        ref.append({k: a[k].clone() for k in ("active_idx", "n_active", "target_pos", "loss_per_sample", "loss_mean", "dX")})
    Wm2, Wb2 = W_bf.float(), W_bf.clone()
    act, n, tp, st = ks.knn_select_active(ys[0], graph, C, M)
    cur = dict(active_idx=act, n_active=n, target_pos=tp)
    other = {k: torch.empty_like(v) for k, v in cur.items()}
    for t in range(3):
        print(f"[case] {name}: step {t} of the headline loop, A={int(ref[t]['n_active'].item())}", flush=True)
        b, _ = ks.knn_softmax_fwd_bwd_update_selected_next(Wm2, Wb2, X_bf, cur["active_idx"], cur["n_active"], cur["target_pos"],
                                                           ys[t + 1], graph, scale, gs, alpha, next_out=other, unit_rows=True,
                                                           trusted_list=True)
        torch.cuda.synchronize()
        assert int(b["dev_status"].item()) == 0
        assert torch.equal(cur["active_idx"], ref[t]["active_idx"]) and torch.equal(cur["target_pos"], ref[t]["target_pos"])
        assert torch.equal(b["loss_per_sample"], ref[t]["loss_per_sample"]) and torch.equal(b["dX"], ref[t]["dX"])
        assert torch.equal(b["loss_mean"], ref[t]["loss_mean"])
        cur, other = other, cur
    assert torch.equal(Wm1, Wm2) and torch.equal(Wb1, Wb2)
    act3, n3, tp3, _ = ks.knn_select_active(ys[3], graph, C, M)
    torch.cuda.synchronize()
    assert torch.equal(cur["active_idx"], act3) and torch.equal(cur["n_active"], n3) and torch.equal(cur["target_pos"], tp3)
