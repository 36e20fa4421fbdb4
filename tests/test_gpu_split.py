"""GPU parity of the softmax split over the nodes of the model-parallel layer (Section 3.1 steps 3-5): each node's
statistics against the oracle's, each node's gradients against the oracle's given the combined statistics, and the
whole thing (all nodes run one after the other on the one GPU, the exchange done with a few tensor operations
standing in for the all-reduce) against the oracle's softmax on one GPU.  Both softmax modes, the three matrix
engines, nodes without any of the batch's classes, random fill-up, and a node of the headline shard's size."""
import numpy as np
import pytest
import torch

import synth
from gradcheck import GRAD_RTOL, check_step_grads

pytestmark = pytest.mark.gpu

LOSS_RTOL = 1e-3


@pytest.fixture(scope="module")
def ks():
    import paper_2102_06025_amd as ks
    ks.lib()
    assert torch.cuda.is_available(), "these tests need the GPU"
    return ks


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t if dtype is None else t.to(dtype)


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


def mixed_features(seed, W, y, D):
    """Half the batch near its label's row (peaky softmax), half anywhere (losses of O(log A))."""
    X = synth.features_near_labels(seed, W, y, bf16=True)
    B = len(y)
    X[B // 2:] = synth.unit_rows(seed + 1, synth.TID_X, B - B // 2, D, bf16=True)
    return X


def run_split(ks, orc, W, X, y, G, bounds, M, scale, grad_scale, unit_rows, pad=False):
    """All nodes on the GPU and in the oracle; returns per-node results of both."""
    Cg, D = W.shape
    B = len(y)
    Xd, yd, Gd = dev(X, torch.bfloat16), dev(y), dev(G)
    K = G.shape[1]
    nodes = []
    for c0, c1 in zip(bounds[:-1], bounds[1:]):
        C_loc = c1 - c0
        Wd = dev(W[c0:c1], torch.bfloat16)
        counts, offsets, flat, st = ks.knn_graph_compress(Gd, c0, C_loc)
        sel = ks.knn_select_active_csr(yd, counts, offsets, flat, c0, C_loc, K, M, pad_random=pad, pad_seed=c0 + 1)
        s1 = ks.knn_softmax_fwd_stats(Wd, Xd, sel["active_idx"], sel["n_active"], sel["target_pos"], scale,
                                      unit_rows=unit_rows)
        torch.cuda.synchronize()
        assert int(st.item()) == 0 and int(sel["dev_status"].item()) == 0 and int(s1["dev_status"].item()) == 0
        # the oracle's node: its own compression and selection (equal to the GPU's: tested elsewhere, asserted here)
        oc = orc.graph_compress(G, c0, C_loc)
        a, n, _, t = orc.select_active_csr(y, *oc, c0, C_loc, M, pad=pad, seed=c0 + 1)
        assert int(sel["n_active"].item()) == n and np.array_equal(sel["active_idx"].cpu().numpy(), a)
        assert np.array_equal(sel["target_pos"].cpu().numpy(), t)
        nodes.append(dict(c0=c0, c1=c1, Wd=Wd, sel=sel, s1=s1, a=a[:n], t=t, n=n))
    # ---- node statistics
    for nd in nodes:
        if nd["n"] == 0:
            assert bool(torch.isneginf(nd["s1"]["row_max"]).all()) and bool((nd["s1"]["row_sumexp"] == 0).all())
            nd["ostats"] = (np.full(B, -np.inf), np.zeros(B), np.zeros(B))
            continue
        m, l, tz = orc.softmax_node_stats(W[nd["c0"]:nd["c1"]], X, nd["a"], nd["t"], scale)
        nd["ostats"] = (m, l, tz)
        gm = nd["s1"]["row_max"].cpu().numpy().astype(np.float64)
        gl = nd["s1"]["row_sumexp"].cpu().numpy().astype(np.float64)
        gt = nd["s1"]["target_logit"].cpu().numpy().astype(np.float64)
        if unit_rows and W.shape[1] in (128, 256, 512):
            assert (gm == scale).all()                            # fixed reference: the nodes only add their sums
        assert np.abs((gm + np.log(gl)) - (m + np.log(l))).max() <= LOSS_RTOL * max(1.0, np.abs(m + np.log(l)).max())
        assert np.abs(gt - tz).max() <= 1e-4 * scale and (gt[nd["t"] < 0] == 0).all()
    # ---- the exchange (stand-in for the all-reduce of Section 3.1 step 4)
    ms = torch.stack([nd["s1"]["row_max"] for nd in nodes])
    ls = torch.stack([nd["s1"]["row_sumexp"] for nd in nodes])
    Mg = ms.max(dim=0).values
    Sg = (ls * torch.exp(ms - Mg[None, :])).sum(dim=0)
    Tg = torch.stack([nd["s1"]["target_logit"] for nd in nodes]).sum(dim=0)
    oM, oS, oT = orc.combine_node_stats([nd["ostats"] for nd in nodes if nd["n"] > 0])
    # ---- second call on every node
    for nd in nodes:
        s2 = ks.knn_softmax_bwd_from_stats(nd["Wd"], Xd, nd["sel"]["active_idx"], nd["sel"]["n_active"],
                                           nd["sel"]["target_pos"], Mg, Sg, Tg, scale, grad_scale, nd["s1"]["ws"],
                                           unit_rows=unit_rows)
        torch.cuda.synchronize()
        assert int(s2["dev_status"].item()) == 0
        nd["s2"] = s2
        if nd["n"] == 0:
            assert bool((s2["dX"] == 0).all())
            continue
        ref = orc.softmax_node_bwd(W[nd["c0"]:nd["c1"]], X, nd["a"], nd["t"], scale, grad_scale, oM, oS, oT)
        nd["ref"] = ref
        li = s2["loss_per_sample"].cpu().numpy()
        assert np.abs(li - ref["loss_i"]).max() <= LOSS_RTOL * max(1.0, np.abs(ref["loss_i"]).max())
        assert abs(float(s2["loss_mean"].item()) - ref["loss"]) <= LOSS_RTOL * abs(ref["loss"])
        print(f"        node [{nd['c0']},{nd['c1']}): A={nd['n']} owned={(nd['t'] >= 0).sum()}", flush=True)
        # every row of the node's dX contribution and of its dW_A; the softmax denominator is the combined one
        ref["lse"] = oM + np.log(oS)
        check_step_grads(s2["dX"].cpu().numpy(), s2["dW_active"][:nd["n"]].cpu().numpy(), ref,
                         W[nd["c0"]:nd["c1"]][nd["a"]], X, nd["t"], scale, grad_scale, tag=f"node {nd['c0']}")
    return nodes, (oM, oS, oT)


@pytest.mark.parametrize("D,unit_rows,pad", [(512, True, False), (512, False, False), (256, True, True), (128, False, True),
                                             (192, False, False), (192, True, False)])
def test_split_over_four_nodes_against_one_gpu(ks, orc, D, unit_rows, pad):
    Cg, B, K, M, scale, gs = 40_000, 320, 16, 4096, 30.0, 128.0
    print(f"[split] Cg={Cg} D={D} B={B} unit_rows={unit_rows} fill-up={pad}", flush=True)
    W = synth.unit_rows(41, synth.TID_W, Cg, D, bf16=True)
    y = synth.labels_uniform(41, B, Cg)
    y[y >= 30_000] -= 30_000                                      # nobody's class on the last node: no owned labels there
    X = mixed_features(41, W, y, D)
    G = synth.graph_synthetic(41, Cg, K, locality=32)
    bounds = [0, 10_000, 10_300, 30_000, 40_000]
    nodes, (oM, oS, oT) = run_split(ks, orc, W, X, y, G, bounds, M, scale, gs, unit_rows, pad)
    # all nodes together are the softmax of one GPU over the union of their lists
    union = np.concatenate([nd["a"] + nd["c0"] for nd in nodes]).astype(np.int32)
    tpos = np.array([int(np.searchsorted(union, c)) for c in y], dtype=np.int32)
    assert (union[tpos] == y).all()
    ref = orc.knn_softmax_fwd_bwd(W, X, union, tpos, scale, gs)
    assert np.allclose(oM + np.log(oS), ref["lse"], rtol=0, atol=1e-9)
    loss = float(nodes[0]["s2"]["loss_mean"].item())
    assert abs(loss - ref["loss"]) <= LOSS_RTOL * abs(ref["loss"])
    dX = sum(nd["s2"]["dX"].double() for nd in nodes).cpu().numpy()
    dW = np.concatenate([nd["s2"]["dW_active"][:nd["n"]].cpu().numpy() for nd in nodes])
    print(f"        all nodes: A={len(union)} loss={loss:.6f} ref={ref['loss']:.6f}", flush=True)
    check_step_grads(dX, dW, ref, W[union], X, tpos, scale, gs, tag="all nodes")


@pytest.mark.parametrize("unit_rows", [True, False])
def test_split_on_a_node_owning_everything_equals_the_one_call_path(ks, orc, unit_rows):
    cfg = synth.CONFIGS["small"]
    C, D, B, K, M, scale = cfg["C"], cfg["D"], cfg["B"], cfg["K"], cfg["M"], cfg["scale"]
    W = synth.unit_rows(42, synth.TID_W, C, D, bf16=True)
    y = synth.make_labels(cfg)
    X = mixed_features(42, W, y, D)
    G = synth.graph_synthetic(42, C, K)
    Wd, Xd, yd, Gd = dev(W, torch.bfloat16), dev(X, torch.bfloat16), dev(y), dev(G)
    one = ks.knn_softmax_fwd_bwd(Wd, Xd, yd, Gd, M, scale, 128.0, unit_rows=unit_rows)
    s1 = ks.knn_softmax_fwd_stats(Wd, Xd, one["active_idx"], one["n_active"], one["target_pos"], scale, unit_rows=unit_rows)
    s2 = ks.knn_softmax_bwd_from_stats(Wd, Xd, one["active_idx"], one["n_active"], one["target_pos"], s1["row_max"],
                                       s1["row_sumexp"], s1["target_logit"], scale, 128.0, s1["ws"], unit_rows=unit_rows)
    torch.cuda.synchronize()
    assert int(s1["dev_status"].item()) == 0 and int(s2["dev_status"].item()) == 0
    A = int(one["n_active"].item())
    # (one-sweep mode: the one-call path takes the loss from the unrounded exponentials, the split path from the sums
    # the nodes exchange, which are those of the stored, rounded values: up to 2^-9 of the smaller of the two terms)
    assert torch.allclose(s2["loss_per_sample"], one["loss_per_sample"], rtol=1e-3 if unit_rows else 1e-5, atol=1e-5)
    assert rel_fro(s2["dX"].cpu().numpy(), one["dX"].cpu().numpy()) <= 1e-3
    assert rel_fro(s2["dW_active"][:A].cpu().numpy(), one["dW_active"][:A].cpu().numpy()) <= 1e-3


def test_split_flags_a_broken_selection(ks):
    C, D, B, M = 1000, 128, 16, 64
    W = torch.randn(C, D, device="cuda").to(torch.bfloat16)
    X = torch.randn(B, D, device="cuda").to(torch.bfloat16)
    act = torch.arange(M, dtype=torch.int32, device="cuda")
    act[3] = C + 5                                                # not a class of this node
    tp = torch.zeros(B, dtype=torch.int32, device="cuda")
    tp[2] = 40                                                    # beyond the 32 valid entries
    n = torch.tensor([32], dtype=torch.int32, device="cuda")
    s1 = ks.knn_softmax_fwd_stats(W, X, act, n, tp, 10.0)
    torch.cuda.synchronize()
    st = int(s1["dev_status"].item())
    assert st & ks.KS_DEV_BAD_INDEX and st & ks.KS_DEV_BAD_LABEL
    assert bool(torch.isfinite(s1["row_max"]).all())


def test_split_node_of_the_headline_shard_size(ks, orc):
    """One node of four at the headline size (390,625 classes of 1,562,500; D = 512; gathered batch 1,024; M = 32,768
    with the random fill-up, so the softmax runs on 32,768 columns) in the one-sweep mode the benchmark times.  The
    rest of the world is a made-up set of statistics (any values are valid inputs of the second call)."""
    cfg = synth.CONFIGS["shard390k"]
    C_loc, D, B, K, M, scale = cfg["C"], cfg["D"], cfg["B"], cfg["K"], cfg["M"], cfg["scale"]
    Cg, c0, gs = 4 * C_loc, C_loc, 128.0
    print(f"[split] headline node: generating {C_loc} rows, Cg={Cg}", flush=True)
    W, _ = synth.make_WX(cfg)
    y = synth.labels_zipf(0, B, Cg, 1.1)
    own = (y >= c0) & (y < c0 + C_loc)
    X = synth.unit_rows(5, synth.TID_X, B, D, bf16=True)
    X[own] = synth.features_near_labels(5, W, y[own] - c0, bf16=True)     # owned samples near their class
    # the node's compressed lists for the batch's labels only (what the selection reads): an arithmetic pattern
    k = np.arange(K, dtype=np.int64)[None, :]
    rows = np.unique(y).astype(np.int64)
    full = ((rows[:, None] + 1 + (rows[:, None] * 2654435761 + k * 40503) % (Cg - 1)) % Cg)
    counts = np.zeros(Cg, dtype=np.int32)
    lists = [r[(r >= c0) & (r < c0 + C_loc)] - c0 for r in full]
    counts[rows] = [len(r) for r in lists]
    offsets = np.zeros(Cg + 1, dtype=np.int64)
    offsets[1:] = np.cumsum(counts)
    flat = np.concatenate(lists).astype(np.int32)
    a, n, nf, t = orc.select_active_csr(y, counts, offsets, flat, c0, C_loc, M, pad=True, seed=9)
    assert n == M
    Wd, Xd = dev(W, torch.bfloat16), dev(X, torch.bfloat16)
    sel = ks.knn_select_active_csr(dev(y), dev(counts), dev(offsets), dev(flat), c0, C_loc, K, M, pad_random=True, pad_seed=9)
    print(f"[split] first call: found {nf}, filled to {n}, owned labels {int(own.sum())}", flush=True)
    s1 = ks.knn_softmax_fwd_stats(Wd, Xd, sel["active_idx"], sel["n_active"], sel["target_pos"], scale, unit_rows=True)
    torch.cuda.synchronize()
    assert int(s1["dev_status"].item()) == 0 and np.array_equal(sel["active_idx"].cpu().numpy(), a)
    print("[split] oracle: node statistics", flush=True)
    m, l, tz = orc.softmax_node_stats(W, X, a, t, scale)
    gm, gl = s1["row_max"].cpu().numpy().astype(np.float64), s1["row_sumexp"].cpu().numpy().astype(np.float64)
    assert np.abs((gm + np.log(gl)) - (m + np.log(l))).max() <= LOSS_RTOL * np.abs(m + np.log(l)).max()
    assert np.abs(s1["target_logit"].cpu().numpy() - tz).max() <= 1e-4 * scale
    # the other three nodes: sums of the same order as this node's, the targets of the samples it does not own
    rng = np.random.default_rng(1)
    m_rest = np.full(B, 0.35 * scale)
    l_rest = 3.0 * np.exp(m + np.log(l) - m_rest) * rng.uniform(0.5, 1.5, B)
    t_rest = np.where(own, 0.0, 0.3 * scale * rng.uniform(0.5, 1.0, B))
    oM, oS, oT = orc.combine_node_stats([(m, l, tz), (m_rest, l_rest, t_rest)])
    s2 = ks.knn_softmax_bwd_from_stats(Wd, Xd, sel["active_idx"], sel["n_active"], sel["target_pos"],
                                       dev(oM.astype(np.float32)), dev(oS.astype(np.float32)), dev(oT.astype(np.float32)),
                                       scale, gs, s1["ws"], unit_rows=True)
    torch.cuda.synchronize()
    assert int(s2["dev_status"].item()) == 0
    print("[split] oracle: node backward", flush=True)
    ref = orc.softmax_node_bwd(W, X, a, t, scale, gs, oM.astype(np.float32), oS.astype(np.float32), oT.astype(np.float32))
    assert abs(float(s2["loss_mean"].item()) - ref["loss"]) <= LOSS_RTOL * abs(ref["loss"])
    print(f"        A={n} loss={float(s2['loss_mean'].item()):.6f} ref={ref['loss']:.6f}", flush=True)
    ref["lse"] = oM.astype(np.float32).astype(np.float64) + np.log(oS.astype(np.float32).astype(np.float64))
    check_step_grads(s2["dX"].cpu().numpy(), s2["dW_active"][:n].cpu().numpy(), ref, W[a[:n]], X, t, scale, gs,
                     tag="headline node")


@pytest.mark.parametrize("Cg,D,K,B,M,P,pad,trusted,unit_rows", [
    (40_000, 128, 16, 128, 2048, 4, False, False, True), (40_000, 128, 16, 128, 2048, 4, True, True, True),
    (9_000, 256, 8, 64, 400, 3, True, False, False), (1_600_000, 64, 8, 96, 1024, 4, False, True, True)])
def test_node_loop_with_the_next_selection_inside_the_second_call(ks, Cg, D, K, B, M, P, pad, trusted, unit_rows):
    """One node of a P-node layer over three batches: knn_softmax_fwd_stats + knn_softmax_bwd_from_stats_next (the next
    batch's selection on the compressed graph inside the second call's launches, with and without the fill-up, the
    list in place or trusted and alternating) against knn_select_active_csr + the two plain calls: lists, counts,
    losses, dX and dW_active bit for bit.  The last case is a node of 400,000 classes (the selection follows the step)."""
    rng = np.random.default_rng(Cg + D)
    c0, C_loc = Cg // P, Cg // P
    W = synth.unit_rows(3, synth.TID_W, C_loc, D, bf16=True)
    X = synth.unit_rows(3, synth.TID_X, B, D, bf16=True)
    c = np.arange(Cg, dtype=np.int64)[:, None]
    k = np.arange(K, dtype=np.int64)[None, :]
    G = ((c + 1 + (c * 2654435761 + k * 40503) % (Cg - 1)) % Cg).astype(np.int32)
    Wd, Xd, Gd = dev(W, torch.bfloat16), dev(X, torch.bfloat16), dev(G)
    counts, offsets, flat, st = ks.knn_graph_compress(Gd, c0, C_loc)
    ys = [dev(rng.integers(0, Cg, B).astype(np.int32)) for _ in range(4)]
    scale, gs = 30.0, 16.0

    def exchange(s1):  # stand-in for the all-reduce: the same on both sides
        return s1["row_max"].clone(), s1["row_sumexp"] * 4.0, s1["target_logit"].clone()

    ref = []
    for t in range(3):
        sel = ks.knn_select_active_csr(ys[t], counts, offsets, flat, c0, C_loc, K, M, pad_random=pad, pad_seed=100 + t)
        s1 = ks.knn_softmax_fwd_stats(Wd, Xd, sel["active_idx"], sel["n_active"], sel["target_pos"], scale, unit_rows=unit_rows)
        gm, gsum, gtz = exchange(s1)
        s2 = ks.knn_softmax_bwd_from_stats(Wd, Xd, sel["active_idx"], sel["n_active"], sel["target_pos"], gm, gsum, gtz, scale, gs,
                                           s1["ws"], unit_rows=unit_rows)
        torch.cuda.synchronize()
        assert int(sel["dev_status"].item()) == 0 and int(s2["dev_status"].item()) == 0
        ref.append((sel, s2))
    sel3 = ks.knn_select_active_csr(ys[3], counts, offsets, flat, c0, C_loc, K, M, pad_random=pad, pad_seed=103)
    first = ks.knn_select_active_csr(ys[0], counts, offsets, flat, c0, C_loc, K, M, pad_random=pad, pad_seed=100)
    cur = dict(active_idx=first["active_idx"], n_active=first["n_active"], n_found=first["n_found"].clone(),
               target_pos=first["target_pos"])
    other = {k_: torch.empty_like(v) for k_, v in cur.items()}
    ws = torch.empty(ks.knn_softmax_split_next_workspace(C_loc, D, B, K, M), dtype=torch.uint8, device="cuda")
    for t in range(3):
        print(f"[case] node step {t}: Cg={Cg} D={D} pad={pad} trusted={trusted}", flush=True)
        sel_ref, s2_ref = ref[t]
        torch.cuda.synchronize()
        assert torch.equal(cur["active_idx"], sel_ref["active_idx"]) and torch.equal(cur["n_active"], sel_ref["n_active"])
        assert torch.equal(cur["target_pos"], sel_ref["target_pos"]) and torch.equal(cur["n_found"], sel_ref["n_found"])
        s1 = ks.knn_softmax_fwd_stats(Wd, Xd, cur["active_idx"], cur["n_active"], cur["target_pos"], scale, unit_rows=unit_rows,
                                      ws=ws, trusted_list=trusted)
        gm, gsum, gtz = exchange(s1)
        nxt = other if trusted else cur
        s2, _ = ks.knn_softmax_bwd_from_stats_next(Wd, Xd, cur["active_idx"], cur["n_active"], cur["target_pos"], gm, gsum, gtz, scale,
                                                   gs, ws, ys[t + 1], counts, offsets, flat, c0, K, next_out=nxt, pad_random=pad,
                                                   pad_seed=100 + t + 1, unit_rows=unit_rows, trusted_list=trusted)
        torch.cuda.synchronize()
        assert int(s2["dev_status"].item()) == 0
        n = int(sel_ref["n_active"].item())
        assert torch.equal(s2["loss_per_sample"], s2_ref["loss_per_sample"]) and torch.equal(s2["dX"], s2_ref["dX"])
        assert torch.equal(s2["dW_active"][:n], s2_ref["dW_active"][:n])
        if trusted:
            cur, other = other, cur
    torch.cuda.synchronize()
    assert torch.equal(cur["active_idx"], sel3["active_idx"]) and torch.equal(cur["n_active"], sel3["n_active"])
    assert torch.equal(cur["target_pos"], sel3["target_pos"]) and torch.equal(cur["n_found"], sel3["n_found"])
    assert int(st.item()) == 0
