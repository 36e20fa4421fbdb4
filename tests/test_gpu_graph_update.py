"""GPU parity of one hop of the distributed graph build (Section 3.2.2): the node's lists after a visiting shard has
been merged in, bit for bit against the CPU oracle (ids and fp64 similarities), hop by hop and after all shards
have visited (= the brute-force graph of the whole problem, = what knn_graph_build gives on one GPU)."""
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


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t if dtype is None else t.to(dtype)


def empty_lists(n, K):
    return (torch.full((n, K), -1, dtype=torch.int32, device="cuda"),
            torch.full((n, K), -np.inf, dtype=torch.float64, device="cuda"))


def run_node(ks, orc, W, bf16, K, shards, node, order, check_hops):
    """All shards visit `node` in `order`; returns the GPU's final lists (and checks every hop when asked)."""
    a, b = shards[node]
    cast = (lambda x: dev(x, torch.bfloat16)) if bf16 else dev
    Wl = cast(W[a:b])
    g, s = empty_lists(b - a, K)
    eg = np.full((b - a, K), -1, dtype=np.int32)
    es = np.full((b - a, K), -np.inf)
    for v in order:
        va, vb = shards[v]
        st = ks.knn_graph_update(Wl, cast(W[va:vb]), a, va, g, s)
        torch.cuda.synchronize()
        assert int(st.item()) == 0
        if check_hops:
            eg, es = orc.graph_update(W[a:b], W[va:vb], a, va, eg, es)
            assert np.array_equal(g.cpu().numpy(), eg), f"node {node}: lists differ after shard {v}"
            assert np.array_equal(s.cpu().numpy(), es), f"node {node}: similarities differ after shard {v}"
    return g, s


@pytest.mark.parametrize("C,D,K,bf16,bounds", [
    (3000, 128, 8, True, [0, 1000, 1001, 2200, 3000]),      # stationary-operand recall, a one-row shard
    (3000, 128, 8, False, [0, 1500, 3000]),                 # fp32 input: 16-bit copies for the recall, fp32 rows for the merge
    (2500, 512, 32, True, [0, 700, 2500]),
    (2000, 96, 16, True, [0, 1200, 2000]),                  # generic recall tile
    (2000, 192, 64, True, [0, 900, 2000]),                  # asynchronous recall tile, k' = 128
    (1500, 256, 100, True, [0, 800, 1500]),                 # k' = 256
])
def test_hops_over_all_shards_give_the_exact_graph(ks, orc, C, D, K, bf16, bounds):
    print(f"[hop] C={C} D={D} K={K} bf16={bf16} shards={bounds}", flush=True)
    W = synth.clustered_rows(7, C, D, n_centres=50, noise=0.4, bf16=bf16)
    W[17] = W[3]                                                  # duplicate rows: ties decided by the id
    W[C - 5] = W[3]
    G, S = orc.graph_bruteforce(W, K)
    shards = list(zip(bounds[:-1], bounds[1:]))
    n = len(shards)
    for node in range(n):
        order = [(node + 1 + t) % n for t in range(n)]            # the ring: the own shard comes last
        g, s = run_node(ks, orc, W, bf16, K, shards, node, order, check_hops=(node == 0))
        a, b = shards[node]
        assert np.array_equal(g.cpu().numpy(), G[a:b]) and np.array_equal(s.cpu().numpy(), S[a:b])
        # a shard that visits again changes nothing
        cast = (lambda x: dev(x, torch.bfloat16)) if bf16 else dev
        g2, s2 = g.clone(), s.clone()
        ks.knn_graph_update(cast(W[a:b]), cast(W[shards[0][0]:shards[0][1]]), a, shards[0][0], g2, s2)
        torch.cuda.synchronize()
        assert torch.equal(g2, g) and torch.equal(s2, s)
    # one GPU that owns everything gives the same lists
    Wd = dev(W, torch.bfloat16) if bf16 else dev(W)
    gb, sb = ks.knn_graph_build(Wd, K, want_sims=True)
    torch.cuda.synchronize()
    assert np.array_equal(gb.cpu().numpy(), G) and np.array_equal(sb.cpu().numpy(), S.astype(np.float32))


def test_hop_with_many_equal_rows_and_short_shards(ks, orc):
    """More copies of a row in the visiting shard than the recall pass keeps (the certificate fails and the row is
    merged against every visiting row), and shards with fewer rows than K (empty slots stay -1 / -inf)."""
    C, D, K = 1200, 128, 16
    W = synth.unit_rows(9, synth.TID_W, C, D, bf16=True)
    W[600:900] = W[5]                                             # 300 copies of row 5 in the second shard
    shards = [(0, 10), (10, 600), (600, 1200)]
    for node in (0, 2):
        a, b = shards[node]
        g, s = run_node(ks, orc, W, True, K, shards, node, [0, 2, 1], check_hops=True)
        G, S = orc.graph_bruteforce(W, K, np.arange(a, b, dtype=np.int32))
        assert np.array_equal(g.cpu().numpy(), G) and np.array_equal(s.cpu().numpy(), S)
    # only the ten-row shard has visited: nine neighbours, seven empty slots
    Wl = dev(W[0:10], torch.bfloat16)
    g, s = empty_lists(10, K)
    ks.knn_graph_update(Wl, Wl, 0, 0, g, s)
    torch.cuda.synchronize()
    gh, sh = g.cpu().numpy(), s.cpu().numpy()
    assert (gh[:, 9:] == -1).all() and np.isneginf(sh[:, 9:]).all() and (gh[:, :9] >= 0).all()
    eg, es = orc.graph_update(W[0:10], W[0:10], 0, 0, np.full((10, K), -1, dtype=np.int32), np.full((10, K), -np.inf))
    assert np.array_equal(gh, eg) and np.array_equal(sh, es)


def test_hop_at_the_headline_shard_size(ks, orc):
    """The node owns the headline shard (390,625 rows, D = 512, K = 32); its own shard and one more of the same size
    visit.  Sampled rows against the oracle's brute force over both shards; properties on all rows."""
    cfg = synth.CONFIGS["shard390k"]
    C, D, K = cfg["C"], cfg["D"], cfg["K"]
    print(f"[hop] headline shard: generating 2 x {C} rows", flush=True)
    W0 = synth.unit_rows(0, synth.TID_W, C, D, bf16=True)
    W1 = synth.unit_rows(1, synth.TID_W, C, D, bf16=True)
    Wl, Wv = dev(W0, torch.bfloat16), dev(W1, torch.bfloat16)
    g, s = empty_lists(C, K)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    print("[hop] visiting shard, then the own shard", flush=True)
    ev[0].record()
    ks.knn_graph_update(Wl, Wv, 0, C, g, s)
    ev[1].record()
    ks.knn_graph_update(Wl, Wl, 0, 0, g, s)
    ev[2].record()
    torch.cuda.synchronize()
    print(f"        hops took {ev[0].elapsed_time(ev[1]):.1f} ms and {ev[1].elapsed_time(ev[2]):.1f} ms", flush=True)
    rng = np.random.default_rng(3)
    rows = np.unique(np.concatenate([rng.integers(0, C, 96), [0, C - 1]])).astype(np.int32)
    print(f"[hop] oracle: brute force of {len(rows)} rows over 2 x {C}", flush=True)
    G, S = orc.graph_bruteforce(np.concatenate([W0, W1]), K, rows)
    sel = torch.from_numpy(rows.astype(np.int64)).cuda()
    assert np.array_equal(g[sel].cpu().numpy(), G) and np.array_equal(s[sel].cpu().numpy(), S)
    ar = torch.arange(C, device="cuda", dtype=torch.int32)[:, None]
    assert bool(((g >= 0) & (g < 2 * C) & (g != ar)).all())
    srt = torch.sort(g, dim=1).values
    assert bool((srt[:, 1:] != srt[:, :-1]).all()) and bool((s[:, 1:] <= s[:, :-1]).all())
    assert bool((g >= C).any()) and bool((g < C).any())           # neighbours from both shards
