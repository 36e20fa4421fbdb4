"""GPU parity of one node of the sharded layer (Section 3.2.3 and the fill-up branch of Algorithm 1): graph
compression, selection on the compressed graph with labels of other nodes' classes, random fill-up to M.  All
outputs are integers and are compared bit for bit with the CPU oracle, on both selection paths (class bitmap in
LDS for nodes of up to 393,216 classes, score table in memory beyond) and at the size of the headline shard."""
import numpy as np
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ks():
    import paper_2102_06025_amd as ks
    ks.lib()
    assert torch.cuda.is_available(), "these tests need the GPU"
    return ks


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def arithmetic_graph(Cg, K):
    """K distinct pseudo-random neighbours per class, none the class itself, spread over the whole id range."""
    c = np.arange(Cg, dtype=np.int64)[:, None]
    k = np.arange(K, dtype=np.int64)[None, :]
    return ((c + 1 + (c * 2654435761 + k * 40503) % (Cg - 1)) % Cg).astype(np.int32)


def compress_both(ks, orc, G, c0, C_loc):
    counts, offsets, flat, st = ks.knn_graph_compress(dev(G), c0, C_loc)
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    ec, eo, ef = orc.graph_compress(G, c0, C_loc)
    assert np.array_equal(counts.cpu().numpy(), ec)
    assert np.array_equal(offsets.cpu().numpy(), eo)
    assert np.array_equal(flat.cpu().numpy(), ef)
    return (counts, offsets, flat), (ec, eo, ef)


@pytest.mark.parametrize("Cg,K,c0,C_loc,empty", [(37, 5, 10, 1, 0.2), (5000, 16, 0, 5000, 0.0), (5000, 16, 1250, 1250, 0.1),
                                                  (100_000, 7, 99_000, 1000, 0.3), (1_200_000, 8, 200_000, 500_000, 0.0),
                                                  (3001, 32, 700, 1500, 0.2), (2500, 64, 0, 1000, 0.1), (1030, 1, 5, 600, 0.3),
                                                  (70_001, 2, 30_000, 20_000, 0.5), (9000, 4, 8999, 1, 0.0)])
def test_graph_compress(ks, orc, Cg, K, c0, C_loc, empty):
    print(f"[csr] compress Cg={Cg} K={K} node=[{c0},{c0 + C_loc}) empty={empty}", flush=True)
    G = synth.graph_synthetic(1, Cg, K, locality=64, empty_frac=empty) if Cg <= 100_000 else arithmetic_graph(Cg, K)
    compress_both(ks, orc, G, c0, C_loc)


def test_graph_compress_flags_short_array_and_bad_ids(ks):
    Cg, K = 3000, 8
    G = arithmetic_graph(Cg, K)
    Gd = dev(G)
    counts = torch.empty(Cg, dtype=torch.int32, device="cuda")
    offsets = torch.empty(Cg + 1, dtype=torch.int64, device="cuda")
    ws = torch.empty(4096, dtype=torch.uint8, device="cuda")
    st = torch.zeros(1, dtype=torch.int32, device="cuda")
    flat = torch.full((100,), -7, dtype=torch.int32, device="cuda")
    import ctypes as ct
    p = lambda t: ct.c_void_p(t.data_ptr())
    rc = ks.lib().knn_graph_compress(p(Gd), ct.c_int64(Cg), ct.c_int(K), ct.c_int64(0), ct.c_int64(1500), p(counts), p(offsets),
                                     p(flat), ct.c_int64(100), p(ws), ct.c_size_t(ws.numel()), p(st), None)
    torch.cuda.synchronize()
    assert rc == 0 and int(st.item()) & ks.KS_DEV_BAD_COUNT
    total = int(offsets[Cg].item())
    assert total == int(((G >= 0) & (G < 1500)).sum()) and total > 100
    f = flat.cpu().numpy()
    o = offsets.cpu().numpy()
    fits = int(np.searchsorted(o, 100, side="right")) - 1         # lists that end inside the short array were written
    assert (f[:o[fits]] >= 0).all() and (f[o[fits]:] == -7).all()
    G[5, 3] = Cg + 9
    _, _, _, st2 = ks.knn_graph_compress(dev(G), 0, 1500)
    torch.cuda.synchronize()
    assert int(st2.item()) & ks.KS_DEV_BAD_GRAPH_ID


def select_both(ks, orc, labels, dev_csr, cpu_csr, c0, C_loc, K_max, M, pad=False, seed=0):
    out = ks.knn_select_active_csr(dev(labels), *dev_csr, c0, C_loc, K_max, M, pad_random=pad, pad_seed=seed)
    torch.cuda.synchronize()
    assert int(out["dev_status"].item()) == 0
    a, n, nf, t = orc.select_active_csr(labels, *cpu_csr, c0, C_loc, M, pad=pad, seed=seed)
    assert int(out["n_active"].item()) == n and int(out["n_found"].item()) == nf
    assert np.array_equal(out["active_idx"].cpu().numpy(), a)
    assert np.array_equal(out["target_pos"].cpu().numpy(), t)
    return a, n, nf, t


@pytest.mark.parametrize("Cg,K,B,P", [(100_000, 16, 256, 4), (20_000, 32, 512, 3), (1_600_000, 16, 1024, 2)])
def test_selection_on_compressed_graph(ks, orc, Cg, K, B, P):
    """Every node of a P-node layer, with and without a cut, with and without the fill-up.  The last case has
    nodes of 800,000 classes (score table in memory), the others use the bitmap in LDS."""
    G = synth.graph_synthetic(2, Cg, K, locality=64, empty_frac=0.05) if Cg <= 100_000 else arithmetic_graph(Cg, K)
    labels = synth.labels_uniform(2, B, Cg)
    for p in range(P):
        c0, C_loc = p * Cg // P, (p + 1) * Cg // P - p * Cg // P
        print(f"[csr] select Cg={Cg} K={K} B={B} node {p}/{P}", flush=True)
        d, c = compress_both(ks, orc, G, c0, C_loc)
        a, n, nf, t = select_both(ks, orc, labels, d, c, c0, C_loc, K, 16384)          # no cut
        assert n == nf and (t == -1).sum() == ((labels < c0) | (labels >= c0 + C_loc)).sum()
        m_cut = max(B, n // 3)
        a2, n2, _, _ = select_both(ks, orc, labels, d, c, c0, C_loc, K, m_cut)         # the cut bites
        assert n2 == m_cut
        a3, n3, nf3, _ = select_both(ks, orc, labels, d, c, c0, C_loc, K, 16384, pad=True, seed=0x1234_5678_9ABC_DEF0 + p)
        assert n3 == min(16384, C_loc) and nf3 == n
        select_both(ks, orc, labels, d, c, c0, C_loc, K, m_cut, pad=True, seed=3)      # nothing to fill


def test_selection_on_a_node_owning_everything_equals_the_dense_entry_point(ks, orc):
    cfg = synth.CONFIGS["small"]
    C, K, B, M = cfg["C"], cfg["K"], cfg["B"], cfg["M"]
    G = arithmetic_graph(C, K)
    labels = synth.make_labels(cfg)
    Gd, yd = dev(G), dev(labels)
    counts, offsets, flat, _ = ks.knn_graph_compress(Gd, 0, C)
    for m in (M, 1024):
        a = ks.knn_select_active_csr(yd, counts, offsets, flat, 0, C, K, m)
        b_idx, b_n, b_pos, _ = ks.knn_select_active(yd, Gd, C, m)
        torch.cuda.synchronize()
        assert torch.equal(a["active_idx"], b_idx) and torch.equal(a["target_pos"], b_pos)
        assert int(a["n_active"].item()) == int(b_n.item())


def test_fill_up_small_nodes_and_seeds(ks, orc):
    Cg, K, B = 4000, 8, 50
    G = synth.graph_synthetic(8, Cg, K, locality=16)
    labels = synth.labels_uniform(8, B, Cg)
    for c0, C_loc, M in [(1000, 1500, 256), (1000, 1500, 1500), (1000, 1500, 3000), (3999, 1, 64), (0, 2, 64), (10, 3, 64)]:
        print(f"[csr] fill-up node=[{c0},{c0 + C_loc}) M={M}", flush=True)
        d, c = compress_both(ks, orc, G, c0, C_loc)
        sets = []
        for seed in (0, 1, 2 ** 63 + 5):
            a, n, nf, _ = select_both(ks, orc, labels, d, c, c0, C_loc, K, M, pad=True, seed=seed)
            assert n == min(M, C_loc)
            sets.append(tuple(a[:n].tolist()))
        if nf + 8 < min(M, C_loc) < C_loc:
            assert len(set(sets)) == 3                            # another seed, another sample


def test_selection_flags_lists_longer_than_promised(ks, orc):
    Cg, K, B = 2000, 8, 32
    G = arithmetic_graph(Cg, K)
    labels = synth.labels_uniform(4, B, Cg)
    counts, offsets, flat, _ = ks.knn_graph_compress(dev(G), 0, Cg)
    out = ks.knn_select_active_csr(dev(labels), counts, offsets, flat, 0, Cg, K - 1, 1024)    # lists hold K entries
    torch.cuda.synchronize()
    assert int(out["dev_status"].item()) & ks.KS_DEV_BAD_COUNT
    bad = offsets.clone()
    bad[int(labels[0])] = flat.numel() - 2                        # a list that runs past the end of the array
    out = ks.knn_select_active_csr(dev(labels), counts, bad, flat, 0, Cg, K, 1024)
    torch.cuda.synchronize()
    assert int(out["dev_status"].item()) & ks.KS_DEV_BAD_COUNT
    out = ks.knn_select_active_csr(dev(np.array([5, Cg], dtype=np.int32)), counts, offsets, flat, 0, Cg, K, 1024)
    torch.cuda.synchronize()
    assert int(out["dev_status"].item()) & ks.KS_DEV_BAD_LABEL


def test_node_of_the_headline_shard_size(ks, orc):
    """One node of four: 1,562,500 classes in all, the node owns 390,625 (the headline shard); K = 32 neighbours per
    class spread over all nodes, a global batch of 1,024 Zipf labels, M = 32,768 with the fill-up."""
    cfg = synth.CONFIGS["shard390k"]
    C_loc, K, B, M = cfg["C"], cfg["K"], cfg["B"], cfg["M"]
    Cg, c0 = 4 * C_loc, C_loc
    print(f"[csr] headline node: Cg={Cg} node=[{c0},{c0 + C_loc}) K={K} B={B} M={M}", flush=True)
    G = arithmetic_graph(Cg, K)
    labels = synth.labels_zipf(0, B, Cg, 1.1)
    d, c = compress_both(ks, orc, G, c0, C_loc)
    assert abs(c[0].mean() - K / 4) < 0.1
    a, n, nf, t = select_both(ks, orc, labels, d, c, c0, C_loc, K, M)
    a2, n2, nf2, t2 = select_both(ks, orc, labels, d, c, c0, C_loc, K, M, pad=True, seed=77)
    print(f"        found {nf} classes, filled up to {n2}; {int((t >= 0).sum())} of {B} labels owned", flush=True)
    assert n2 == M and nf2 == nf == n
    # twice the same call, the same bits
    o1 = ks.knn_select_active_csr(dev(labels), *d, c0, C_loc, K, M, pad_random=True, pad_seed=77)
    o2 = ks.knn_select_active_csr(dev(labels), *d, c0, C_loc, K, M, pad_random=True, pad_seed=77)
    torch.cuda.synchronize()
    assert torch.equal(o1["active_idx"], o2["active_idx"]) and torch.equal(o1["target_pos"], o2["target_pos"])
