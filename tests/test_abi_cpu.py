"""CPU-side checks of the C-ABI library: it loads without a GPU, exports every symbol the header declares,
sizes its workspaces sensibly and rejects bad arguments before touching the device."""
import ctypes as ct
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "knnsoftmax.h")


@pytest.fixture(scope="module")
def ks():
    import paper_2102_06025_amd as ks
    if not os.path.exists(ks.lib_path()):
        from paper_2102_06025_amd.build import build
        build()
    ks.lib()
    return ks


def _declared_functions():
    src = open(HEADER).read() + open(os.path.join(ROOT, "include", "grad_topk.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(ks_version|ks_peak_mfma|ks_peak_copy|[a-z_]+(?:_workspace|_build|_active|_rows|_fwd_bwd|_grad|_normalized|_csr|_compress|_update|_stats|_profiled|_plan|_select|_static|_selected|_next))\s*\(", src)))


def test_header_symbols_are_exported(ks):
    names = _declared_functions()
    assert {"knn_graph_build", "knn_softmax_fwd_bwd", "apply_weight_grad", "apply_weight_grad_normalized",
            "knn_normalize_rows", "knn_norm_backward_rows", "grad_topk_plan", "grad_topk_workspace",
            "grad_topk_select", "knn_select_active_static", "knn_softmax_fwd_bwd_update_selected_next",
            "knn_softmax_selected_next_workspace", "knn_softmax_bwd_from_stats_next", "knn_softmax_split_next_workspace"} <= set(names)
    L = ks.lib()
    for n in names:
        assert hasattr(L, n), f"{n} declared in the header but not exported"
    assert "gfx950" in ks.ks_version()


def test_index_and_weight_types_match_the_papers_byte_counts():
    # Section 3.1: 100 M x 512 weights are "about 190 GB" => 4-byte weights; Section 3.2.3: a 100 M x 1000 graph is
    # "about 372 GB" => 4-byte ids (tests/golden/paper_sizes.txt)
    gold = dict(l.split()[:2] for l in open(os.path.join(ROOT, "tests", "golden", "paper_sizes.txt")) if l[0] != "#")
    assert int(100e6 * 512 * 4 / 2 ** 30) == int(gold["fc_weight_GiB"])
    assert int(100e6 * 1000 * 4 / 2 ** 30) == int(gold["graph_GiB"])
    src = open(HEADER).read()
    assert "int32_t *graph" in src and "float *W_master" in src


def test_workspace_sizes(ks):
    a = ks.knn_softmax_workspace(390625, 512, 1024, 32, 32768)
    # at least the transposed logit gradient (bf16; the logits themselves are never stored) and one set of
    # dX partial sums; far less than logits + gradient in fp32 would take
    assert a >= 1024 * 32768 * 2 + 1024 * 512 * 4
    assert a < 1024 * 32768 * 4
    assert ks.knn_softmax_workspace(100, 33, 4, 2, 8) == 0          # D % 32 != 0
    assert ks.knn_graph_build_workspace(1000, 128, 200, 0) == 0     # K too large
    assert ks.knn_graph_build_workspace(390625, 512, 32, 0) < 10 << 30   # 2,048 candidate slots per row, and the logs
    assert ks.apply_weight_grad_workspace(1000, 128, 100, 1) <= 256
    assert ks.apply_weight_grad_workspace(1000, 128, 100, 0) >= 128 * 8


def test_argument_errors_are_reported_before_any_launch(ks):
    L = ks.lib()
    null = ct.c_void_p(0)
    one = ct.c_void_p(256)  # never dereferenced: validation fails first
    i64, i, f, sz = ct.c_int64, ct.c_int, ct.c_float, ct.c_size_t

    def fwd(C=1000, D=128, B=8, K=4, M=64, W=one, ws_bytes=1 << 30):
        return L.knn_softmax_fwd_bwd(W, one, one, one, i64(C), i(D), i(B), i(K), i(M), f(30.0), f(1.0), ct.c_uint32(0),
                                     one, one, one, one, one, one, one, one, sz(ws_bytes), null, null)

    assert fwd(W=null) == ks.KS_INVALID_ARG
    assert fwd(D=100) == ks.KS_INVALID_ARG            # D % 32
    assert fwd(B=65) == ks.KS_INVALID_ARG             # B > M
    assert fwd(K=64) == ks.KS_INVALID_ARG             # K + 1 > M
    assert fwd(C=0) == ks.KS_INVALID_ARG
    assert fwd(ws_bytes=1024) == ks.KS_WORKSPACE_TOO_SMALL

    def upd_step(Wm=one, dW=null, D=128):
        return L.knn_softmax_fwd_bwd_update(Wm, one, one, one, one, i64(1000), i(D), i(8), i(4), i(64), f(30.0), f(1.0),
                                            f(-0.01), ct.c_uint32(0), one, one, one, one, one, one, dW, one, sz(1 << 30),
                                            null, null)

    assert upd_step(Wm=null) == ks.KS_INVALID_ARG
    assert upd_step(D=96) == ks.KS_INVALID_ARG        # the gradient has to be stored on the paths without the fused update

    def graph(C=1000, D=128, K=8, dtype=0, ws_bytes=1 << 40):
        return L.knn_graph_build(one, i(dtype), i64(C), i(D), i(K), one, null, one, sz(ws_bytes), null, null)

    assert graph(K=129) == ks.KS_UNSUPPORTED
    assert graph(C=8, K=8) == ks.KS_UNSUPPORTED       # K > C - 1
    assert graph(dtype=7) == ks.KS_INVALID_ARG
    assert graph(D=72) == ks.KS_INVALID_ARG
    assert graph(ws_bytes=16) == ks.KS_WORKSPACE_TOO_SMALL

    def apply(n_max=10, D=128, sorted_=1, ws=one, ws_bytes=0, Wm=one):
        return L.apply_weight_grad(Wm, one, one, null, i(n_max), one, f(-0.1), i64(1000), i(D), i(sorted_), ws,
                                   sz(ws_bytes), null, null)

    assert apply(Wm=null) == ks.KS_INVALID_ARG
    assert apply(n_max=0) == ks.KS_INVALID_ARG
    assert apply(D=6) == ks.KS_INVALID_ARG
    assert apply(sorted_=0, ws_bytes=8) == ks.KS_WORKSPACE_TOO_SMALL

    def apply_n(n_max=10, D=128, sorted_=1, ws=one, ws_bytes=0, Wm=one):
        return L.apply_weight_grad_normalized(Wm, one, one, one, null, i(n_max), one, f(-0.1), i64(1000), i(D), i(sorted_),
                                              ws, sz(ws_bytes), null, null)

    assert apply_n(Wm=null) == ks.KS_INVALID_ARG
    assert apply_n(D=6) == ks.KS_INVALID_ARG
    assert apply_n(sorted_=0, ws=null) == ks.KS_INVALID_ARG
    assert apply_n(sorted_=0, ws_bytes=8) == ks.KS_WORKSPACE_TOO_SMALL
    assert ks.apply_weight_grad_normalized_workspace(1000, 128, 100, 0) >= 128 * 8 + 128 * 128 * 4

    def csr(Cg=1000, c0=100, C_loc=200, B=8, K=4, M=64, flags=0, ws_bytes=1 << 30, flat=one, flat_len=10):
        return L.knn_select_active_csr(one, one, one, flat, i64(flat_len), i64(Cg), i64(c0), i64(C_loc), i(B), i(K), i(M),
                                       ct.c_uint32(flags), ct.c_uint64(1), one, one, null, one, one, sz(ws_bytes), null, null)

    assert csr(c0=900) == ks.KS_INVALID_ARG           # the node's range sticks out of the problem
    assert csr(B=65) == ks.KS_INVALID_ARG
    assert csr(flags=8) == ks.KS_INVALID_ARG
    assert csr(flat=null) == ks.KS_INVALID_ARG
    assert csr(ws_bytes=16) == ks.KS_WORKSPACE_TOO_SMALL
    assert L.knn_graph_compress(one, i64(1000), i(8), i64(990), i64(20), one, one, null, i64(0), one, sz(1 << 20), null,
                                null) == ks.KS_INVALID_ARG
    assert L.knn_graph_compress(one, i64(1000), i(8), i64(0), i64(20), one, one, null, i64(0), one, sz(0), null,
                                null) == ks.KS_WORKSPACE_TOO_SMALL

    def upd(C_loc=100, C_vis=50, D=128, K=8, lo=0, vo=100, ws_bytes=1 << 40, dtype=0):
        return L.knn_graph_update(one, one, i(dtype), i64(C_loc), i64(C_vis), i(D), i(K), i64(lo), i64(vo), one, one, one,
                                  sz(ws_bytes), null, null)

    assert upd(D=72) == ks.KS_INVALID_ARG
    assert upd(K=129) == ks.KS_UNSUPPORTED
    assert upd(vo=(1 << 31) - 10) == ks.KS_INVALID_ARG    # ids must stay below 2^31
    assert upd(dtype=5) == ks.KS_INVALID_ARG
    assert upd(ws_bytes=64) == ks.KS_WORKSPACE_TOO_SMALL

    def stats(D=128, B=8, M=64, scale=30.0, flags=0, ws_bytes=1 << 30, W=one):
        return L.knn_softmax_fwd_stats(W, one, one, one, one, i64(1000), i(D), i(B), i(M), f(scale), ct.c_uint32(flags), one,
                                       one, one, one, sz(ws_bytes), null, null)

    assert stats(W=null) == ks.KS_INVALID_ARG
    assert stats(D=96) == ks.KS_UNSUPPORTED            # the split runs on the D % 64 == 0 paths
    assert stats(scale=0.0) == ks.KS_INVALID_ARG
    assert stats(flags=2) == ks.KS_INVALID_ARG
    assert stats(ws_bytes=64) == ks.KS_WORKSPACE_TOO_SMALL
    assert L.knn_softmax_bwd_from_stats(one, one, one, one, one, one, one, null, i64(1000), i(128), i(8), i(64), f(30.0),
                                        f(1.0), ct.c_uint32(0), one, one, one, one, one, sz(1 << 30), null,
                                        null) == ks.KS_INVALID_ARG
    assert ks.knn_softmax_split_workspace(1000, 128, 8, 64) > ks.knn_softmax_split_workspace(1000, 96, 8, 64) == 0
    assert L.knn_normalize_rows(one, i(0), i64(4), i(128), null, null, null) == ks.KS_INVALID_ARG   # no output
    assert L.knn_normalize_rows(one, i(3), i64(4), i(128), one, one, null) == ks.KS_INVALID_ARG     # dtype
    assert L.knn_normalize_rows(one, i(0), i64(4), i(6), one, one, null) == ks.KS_INVALID_ARG       # D % 4
    assert L.knn_norm_backward_rows(one, i(1), null, i64(4), i(128), one, null) == ks.KS_INVALID_ARG
    assert L.knn_select_active(one, one, i64(100), i(8), i(4), i(4), one, one, one, one, sz(1 << 20), null,
                               null) == ks.KS_INVALID_ARG  # B > M

    two = ct.c_void_p(512)

    def nxt(labels_next=one, K=4, M=64, flags=0, act_next=two, n_next=two, tp_next=two, ws_bytes=1 << 30, graph=one):
        return L.knn_softmax_fwd_bwd_update_selected_next(one, one, one, one, one, one, i64(1000), i(128), i(8), i(M), f(30.0),
                                                          f(1.0), f(-0.01), ct.c_uint32(flags), one, one, one, null,
                                                          labels_next, graph, i(K), act_next, n_next, tp_next, one,
                                                          sz(ws_bytes), null, null)

    assert nxt(labels_next=null) == ks.KS_INVALID_ARG
    assert nxt(graph=null) == ks.KS_INVALID_ARG
    assert nxt(act_next=null) == ks.KS_INVALID_ARG
    assert nxt(K=64) == ks.KS_INVALID_ARG              # K + 1 > M
    assert nxt(flags=2) == ks.KS_INVALID_ARG           # not a flag of this call
    assert nxt(flags=4, act_next=one) == ks.KS_INVALID_ARG   # a trusted list is read in place: the next one needs its own buffers
    assert nxt(ws_bytes=1024) == ks.KS_WORKSPACE_TOO_SMALL
    assert ks.knn_softmax_selected_next_workspace(1000, 128, 8, 4, 64) >= ks.knn_softmax_selected_workspace(1000, 128, 8, 64) + 8 * 5 * 4
    assert ks.knn_softmax_selected_next_workspace(1000, 100, 8, 4, 64) == 0

    def split_next(labels_next=one, counts=one, K_max=4, c0=100, Cg=2000, sel_flags=0, flags=0, act_next=two, ws_bytes=1 << 30,
                   D=128):
        return L.knn_softmax_bwd_from_stats_next(one, one, one, one, one, one, one, one, i64(1000), i(D), i(8), i(64), f(30.0),
                                                 f(1.0), ct.c_uint32(flags), one, one, one, one, labels_next, counts, one, one,
                                                 i64(10), i64(Cg), i64(c0), i(K_max), ct.c_uint32(sel_flags), ct.c_uint64(1),
                                                 act_next, two, null, two, one, sz(ws_bytes), null, null)

    assert split_next(labels_next=null) == ks.KS_INVALID_ARG
    assert split_next(counts=null) == ks.KS_INVALID_ARG
    assert split_next(c0=1500) == ks.KS_INVALID_ARG          # the node's range sticks out of the problem
    assert split_next(K_max=64) == ks.KS_INVALID_ARG         # K_max + 1 > M
    assert split_next(sel_flags=1) == ks.KS_INVALID_ARG      # only the fill-up flag belongs to the selection
    assert split_next(flags=4, act_next=one) == ks.KS_INVALID_ARG   # trusted list: the next one needs its own buffers
    assert split_next(D=96) == ks.KS_UNSUPPORTED
    assert split_next(ws_bytes=1024) == ks.KS_WORKSPACE_TOO_SMALL
    assert ks.knn_softmax_split_next_workspace(1000, 128, 8, 4, 64) >= ks.knn_softmax_split_workspace(1000, 128, 8, 64) + 8 * 5 * 4


def test_product_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2102_06025_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in text.lower(), f"{fn} mentions the oracle"


# ------------------------------------------------------------------------------------------------
# planning of the layer-wise top-k selection (host logic of include/grad_topk.h)
# ------------------------------------------------------------------------------------------------
def _plan(ks, sizes, k, chunks=0):
    import numpy as np
    offs = np.zeros(len(sizes) + 1, dtype=np.int64)
    offs[1:] = np.cumsum(sizes)
    k = np.asarray(k, dtype=np.int32)
    L = ks.lib()
    args = (offs.ctypes.data_as(ct.c_void_p), k.ctypes.data_as(ct.c_void_p), ct.c_int(len(sizes)), ct.c_int(chunks))
    words = L.grad_topk_plan(*args, ct.c_void_p(0), ct.c_int64(0))
    if words < 0:
        return words, None
    plan = np.zeros(words, dtype=np.int64)
    assert L.grad_topk_plan(*args, plan.ctypes.data_as(ct.c_void_p), ct.c_int64(words)) == words
    return words, plan


NODE = 12   # words of a step record: src, items, k, out, flags, first, tensor begin, tensor size, aux, tree first, tree steps
F_LEAF, F_FINAL, F_THRESH, F_FILTER, F_COUNTED = 1, 2, 4, 8, 16


def _check_plain_tree(np, nodes, n, k, out):
    """nodes: the steps of one tensor's tree of selections, level by level.  Leaves tile the tensor, every inner step reads
    whole lists that earlier steps wrote, no step takes more than 32,768 items, the last one writes the output."""
    src, items, nk, o, flags = nodes.T[:5]
    leaf, final = (flags & F_LEAF) == F_LEAF, (flags & F_FINAL) == F_FINAL
    assert final.sum() == 1 and final[-1] and o[-1] == out and (nk == k).all() and not (flags & (F_THRESH | F_FILTER | F_COUNTED)).any()
    assert (items <= 32768).all() and items[-1] >= k
    ls = np.argsort(src[leaf], kind="stable")
    assert (src[leaf][ls][1:] == (src[leaf] + items[leaf])[ls][:-1]).all() and items[leaf].sum() == n
    keep = np.minimum(items, nk)
    if len(nodes) > 1:
        starts = set(o[~final].tolist())
        assert all(int(x) in starts for x in src[~leaf]) and items[~leaf].sum() == keep[~final].sum()
    return int(leaf.sum())


def test_topk_plan_layout(ks):
    import numpy as np
    import synth
    sizes = synth.resnet50_tensor_sizes()
    k = synth.topk_counts(sizes)
    words, plan = _plan(ks, sizes, k)
    T = len(sizes)
    offs = np.concatenate([[0], np.cumsum(sizes)])
    assert plan[1] == T and plan[4] == k.sum() and plan[5] == sum(sizes)
    n, kk, M, levels = plan[32:32 + 4 * T].reshape(T, 4).T
    assert (n == sizes).all() and (kk == k).all() and (M == -(-n // 32768)).all()
    # tensors of several chunks take the sampled path here (k is a thousandth of n): threshold, filters, final step
    assert (levels[M == 1] == 1).all() and (levels[M > 1] == 3).all() and plan[6] == 3
    n_launched, n_nodes = int(plan[2]), int(plan[7])
    assert words == 32 + 4 * T + NODE * n_nodes and n_launched == (M == 1).sum() + (M[M > 1] + 2).sum()
    nodes = plan[32 + 4 * T:].reshape(n_nodes, NODE)
    src, items, nk, out, flags, first, gbegin, gn, aux, fb_first, fb_count = nodes.T[:11]
    firsts, counts = plan[8:8 + 2 * 3:2], plan[9:9 + 2 * 3:2]
    assert firsts[0] == 0 and (firsts[1:] == np.cumsum(counts)[:-1]).all() and counts.sum() == n_launched
    lev = np.repeat(np.arange(3), counts)
    L = nodes[:n_launched]
    fl = L[:, 4]
    # level 0: one threshold step per sampled tensor; level 1: its filters, first in the level; level 2: the final steps of
    # the sampled paths first, then the tensors of a single step
    assert ((fl[lev == 0] & F_THRESH) != 0).all() and counts[0] == (M > 1).sum()
    assert ((fl[lev == 1] & F_FILTER) != 0).all() and plan[28] == firsts[1] and plan[29] == counts[1] == M[M > 1].sum()
    assert plan[30] == firsts[2] and plan[31] == (M > 1).sum()
    l2 = fl[lev == 2]
    assert ((l2[:plan[31]] & F_COUNTED) != 0).all() and (l2[plan[31]:] == (F_LEAF | F_FINAL)).all()
    # the filters of a tensor tile it; all final steps tile the output; the sampled paths' lists and words do not overlap
    for t in np.nonzero(M > 1)[0]:
        mine = L[(lev == 1) & (L[:, 6] == offs[t])]
        o = np.argsort(mine[:, 0], kind="stable")
        assert mine[o][0, 0] == offs[t] and (mine[o][1:, 0] == (mine[:, 0] + mine[:, 1])[o][:-1]).all() and mine[:, 1].sum() == n[t]
        assert (mine[:, 5] == mine[:, 0] - offs[t]).all() and len(set(mine[:, 8])) == 1 and len(set(mine[:, 3])) == 1
    fin = L[(fl & F_FINAL) != 0]
    assert sorted(fin[:, 3].tolist()) == [0] + np.cumsum(k)[:-1].tolist()
    counted = L[(fl & F_COUNTED) != 0]
    regions = sorted((int(a), int(a) + 2 + 32768) for a in counted[:, 8])
    assert all(b[0] >= a[1] for a, b in zip(regions, regions[1:])) and regions[-1][1] <= plan[3]
    assert (counted[:, 0] == counted[:, 8] + 2).all() and (counted[:, 1] == 32768).all()
    th = L[(fl & F_THRESH) != 0]
    assert (th[:, 2] >= 16).all() and (th[:, 2] <= 512).all() and sorted(th[:, 8].tolist()) == sorted(counted[:, 8].tolist())
    # behind the launched steps: the plain tree of every sampled tensor (what its final step falls back on)
    assert n_nodes - n_launched == counted[:, 10].sum()
    big = n == 512 * 512 * 9   # 72 chunks x 2,359 survivors = 169,848 items: reduced in groups of 13 chunks first
    for c in counted:
        t = int(np.nonzero(offs[:-1] == c[6])[0][0])
        tree = nodes[c[9]:c[9] + c[10]]
        assert c[9] >= n_launched and (tree[:, 6] == offs[t]).all()
        leaves = _check_plain_tree(np, tree, n[t], k[t], c[3])
        assert leaves == M[t] and (len(tree) == 72 + 6 + 1 if big[t] else len(tree) >= M[t] + 1)
    assert ks.lib().grad_topk_workspace(plan.ctypes.data_as(ct.c_void_p)) >= int(plan[3]) * 8
    # forced chunk counts: the paper's two steps (or a deeper tree), no sampled path
    _, p2 = _plan(ks, [100, 10_000], [5, 10], chunks=7)
    assert p2[32 + 2] == 7 and p2[32 + 4 + 2] == 7 and p2[6] == 2 and p2[29] == 0 and p2[31] == 0 and p2[2] == p2[7]
    nodes2 = p2[32 + 8:].reshape(-1, NODE)
    assert nodes2[:7, 1].tolist() == [15] * 6 + [10] and nodes2[7:14, 1].tolist() == [1429] * 6 + [1426]
    _check_plain_tree(np, nodes2[(nodes2[:, 6] == 100)], 10_000, 10, 5)
    _, p3 = _plan(ks, [5], [5], chunks=64)
    assert p3[32 + 2] == 5 and p3[2] == 6 and p3[6] == 2
    # a tensor whose k is large for its size keeps the plain tree even with several chunks
    _, p4 = _plan(ks, [1_000_000], [2000])
    assert p4[29] == 31 and p4[32 + 3] == 3 and p4[32 + 4 + 2] == 33   # threshold = 33rd of the sample: 8,000 items expected
    _, p5 = _plan(ks, [300_000], [4096])
    assert p5[29] == 0 and p5[31] == 0 and p5[32 + 3] >= 2             # three times 16,400 expected items are more than a step takes


@pytest.mark.parametrize("C,D,K,dtype", [(6400, 128, 32, 0), (7000, 128, 8, 0), (8330, 256, 16, 1), (6913, 512, 32, 0),
                                         (25_000, 128, 32, 0), (50_011, 128, 16, 0), (101_000, 256, 32, 0),
                                         (390_625, 512, 32, 0), (393_216, 512, 32, 0), (399_000, 512, 32, 1)])
def test_graph_plan_pairs_every_two_blocks_exactly_once(ks, C, D, K, dtype):
    """The division of work of the graph build that computes every similarity once: every block of 256 rows is some
    workgroup's, and for every two different blocks exactly one of the two workgroups streams the other's rows with both
    sides of the similarity in use; a workgroup's own block is streamed by itself (for its own rows); ranges lie on
    96-row chunk boundaries; the load is even."""
    import numpy as np
    n_wg, _ = ks.knn_graph_build_plan(C, D, K, dtype)
    assert n_wg > 0
    NB = -(-C // 256)
    taken = np.zeros((NB, NB), dtype=np.uint8) if NB <= 512 else None
    pairs = np.zeros(NB, dtype=np.int64)     # blocks paired by each resident block
    seen = np.zeros(NB, dtype=np.int64)
    rows_streamed = []
    for wg in range(n_wg):
        _, p = ks.knn_graph_build_plan(C, D, K, dtype, wg)
        b = p[0]
        if b < 0:
            assert all(p[2 + 2 * q] <= p[1 + 2 * q] for q in range(5))
            continue
        seen[b] += 1
        own_sb = b * 256 // 768
        assert p[1] == own_sb * 768 and p[2] == min(p[1] + 768, C)         # range 0: its own super-block
        n_own = -(-(p[2] - p[1]) // 256)
        assert p[11] < (1 << n_own) and not (p[11] >> (b - own_sb * 3)) & 1
        mine = [own_sb * 3 + k for k in range(n_own) if (p[11] >> k) & 1]
        total = p[2] - p[1]
        for q in range(1, 5):
            first, end = p[1 + 2 * q], p[2 + 2 * q]
            if end <= first:
                continue
            assert first % 768 == 0 and (end % 768 == 0 or end == C) and end <= C
            assert not first <= b * 256 < end                                # never its own rows again
            mine += list(range(first // 256, -(-end // 256)))
            total += end - first
        rows_streamed.append(total)
        assert len(set(mine)) == len(mine)
        pairs[b] = len(mine)
        if taken is not None:
            taken[b, mine] += 1
    assert (seen == 1).all()
    assert pairs.sum() == NB * (NB - 1) // 2                                  # as many pairs as there are
    if taken is not None:
        both = taken + taken.T
        assert (both[~np.eye(NB, dtype=bool)] == 1).all() and (np.diag(taken) == 0).all()
    else:   # large problems: the counts per block (every block is paired NB - 1 times in all) by sampling the relation
        rng = np.random.default_rng(0)
        sets = {}
        for wg in range(n_wg):
            _, p = ks.knn_graph_build_plan(C, D, K, dtype, wg)
            if p[0] >= 0:
                sets[p[0]] = p
        def takes(a, b):
            p = sets[a]
            own_sb = a * 256 // 768
            if b // 3 == own_sb:
                return bool((p[11] >> (b - own_sb * 3)) & 1)
            return any(p[1 + 2 * q] <= b * 256 < p[2 + 2 * q] for q in range(1, 5))
        for a, b in rng.integers(0, NB, (20000, 2)):
            if a != b:
                assert takes(a, b) != takes(b, a)
    # nobody streams much more than half of the rows
    assert max(rows_streamed) <= C / 2 + 12 * 768 and max(rows_streamed) - min(rows_streamed) <= max(0.06 * C, 4 * 768)


def test_graph_plan_is_absent_for_small_problems(ks):
    for C, D, K, dtype in [(6000, 128, 32, 0), (390_625, 192, 32, 0), (390_625, 512, 65, 0), (6000, 256, 16, 1)]:
        assert ks.knn_graph_build_plan(C, D, K, dtype)[0] == 0
    with pytest.raises(ks.KsError):
        ks.knn_graph_build_plan(1, 128, 32, 0)
    with pytest.raises(ks.KsError):
        ks.knn_graph_build_plan(390_625, 512, 32, 0, workgroup=10_000_000)


def test_topk_argument_errors(ks):
    assert _plan(ks, [10], [0])[0] == -ks.KS_INVALID_ARG          # k < 1
    assert _plan(ks, [10], [11])[0] == -ks.KS_INVALID_ARG         # k > n
    assert _plan(ks, [10, 0], [1, 1])[0] == -ks.KS_INVALID_ARG    # an empty tensor
    assert _plan(ks, [100_000], [5000])[0] == -ks.KS_UNSUPPORTED  # k beyond the limit
    L = ks.lib()
    import numpy as np
    junk = np.zeros(64, dtype=np.int64)
    assert L.grad_topk_workspace(junk.ctypes.data_as(ct.c_void_p)) == 0
    one = ct.c_void_p(256)
    assert L.grad_topk_select(one, one, junk.ctypes.data_as(ct.c_void_p), one, one, one, ct.c_size_t(1 << 20), None) == ks.KS_INVALID_ARG
    _, plan = _plan(ks, [100_000], [100])
    ph = plan.ctypes.data_as(ct.c_void_p)
    assert L.grad_topk_select(None, one, ph, one, one, one, ct.c_size_t(1 << 20), None) == ks.KS_INVALID_ARG
    assert L.grad_topk_select(one, one, ph, one, one, one, ct.c_size_t(8), None) == ks.KS_WORKSPACE_TOO_SMALL


def test_bench_refuses_more_than_one_gpu():
    # the benchmark measures one GPU's share; asking for more ends with a message and a non-zero status, before any GPU work
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in (r.stdout + r.stderr)


def test_static_selection_rejects_sizes_beyond_its_scratch_array_before_any_launch(ks):
    """knn_select_active_static: sizes whose scratch need exceeds KS_SELECT_STATIC_BYTES are KS_UNSUPPORTED, bad
    arguments KS_INVALID_ARG; neither touches the device (no GPU here)."""
    L = ks.lib()
    null, one = ct.c_void_p(0), ct.c_void_p(256)
    i64, i = ct.c_int64, ct.c_int

    def sel(C=390_625, B=1024, K=32, M=32_768, labels=one):
        return L.knn_select_active_static(labels, one, i64(C), i(B), i(K), i(M), one, one, one, null, null)

    src = open(HEADER).read()
    limit = int(re.search(r"#define KS_SELECT_STATIC_BYTES \((\d+)u << (\d+)\)", src).group(1)) << 20
    assert limit == ks.binding.KS_SELECT_STATIC_BYTES
    assert ks.knn_select_workspace(390_625, 1024, 32, 32_768) <= limit       # the headline shape fits
    assert ks.knn_select_workspace(1_000_000, 2048, 64, 131_072) > limit
    assert sel(C=1_000_000, B=2048, K=64, M=131_072) == ks.KS_UNSUPPORTED
    assert sel(B=20_000, K=32) == ks.KS_UNSUPPORTED                          # staging array of 20,000 x 33 candidates
    assert sel(labels=null) == ks.KS_INVALID_ARG
    assert sel(B=40_000) == ks.KS_INVALID_ARG                                # B > M


def test_bench_reads_the_traffic_figures_from_the_committed_profile():
    """The `traffic` fields of the benchmark line come from profiles/bench_shard390k_hbm_traffic.txt at run time: the
    parser finds the step's three contraction kernels there, and the figures are the file's own last column."""
    import bench
    t = bench.profiled_traffic()
    assert set(t) == {"logits_gemm", "dx_gemm", "dw_gemm"}
    text = open(bench.TRAFFIC_PROFILE).read()
    for stage, kernel in bench.TRAFFIC_KERNEL.items():
        line = [ln for ln in text.splitlines() if ln.startswith(kernel)][0]
        assert t[stage] == float(line.split()[-1]) * 1e6 and 1e6 < t[stage] < 1e9
    assert bench.profiled_traffic("/nonexistent/file") == {}
