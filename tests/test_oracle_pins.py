"""Pins for the CPU oracle: every oracle function is checked against something that is not its own
formula -- the full-softmax special case (paper Section 3.2: KNN softmax is standard softmax on the
selected columns), a library cross-entropy with autograd in fp64, closed forms, invariants, finite
differences, set-based selection, argsort-based neighbour search with exactly representable
similarities, and a dense index_add."""
import math

import numpy as np
import pytest
import torch

import synth


# --------------------------------------------------------------------------------------------
# softmax / cross-entropy / gradients
# --------------------------------------------------------------------------------------------
def _small_problem(C=2000, D=32, B=16, seed=3):
    W = synth.unit_rows(seed, synth.TID_W, C, D)
    X = synth.unit_rows(seed, synth.TID_X, B, D)
    y = synth.labels_uniform(seed, B, C)
    return W, X, y


def test_knn_softmax_equals_full_softmax_when_lists_span_all_classes(orc):
    # Section 3.2: same result as standard softmax.  K = C-1 (+ the class itself) makes every class active.
    C, D, B = 2000, 32, 16
    W, X, y = _small_problem(C, D, B)
    G = synth.graph_all_others(C)
    active, A, tpos = orc.select_active(y, G, C, M=C)
    assert A == C and (active == np.arange(C)).all() and (tpos == y).all()
    knn = orc.knn_softmax_fwd_bwd(W, X, active[:A], tpos, scale=30.0, grad_scale=2.0)
    full = orc.full_softmax_fwd_bwd(W, X, y, scale=30.0, grad_scale=2.0)
    # same summation order in both functions => bit-equal
    assert knn["loss"] == full["loss"]
    assert (knn["loss_i"] == full["loss_i"]).all()
    assert (knn["dX"] == full["dX"]).all()
    assert (knn["dWA"] == full["dW"]).all()


def _torch_ce(W, X, cols, tgt, scale, grad_scale):
    Wt = torch.tensor(W[cols], dtype=torch.float64, requires_grad=True)
    Xt = torch.tensor(X, dtype=torch.float64, requires_grad=True)
    Z = scale * Xt @ Wt.T
    li = torch.nn.functional.cross_entropy(Z, torch.tensor(tgt, dtype=torch.long), reduction="none")
    loss = li.mean()
    (grad_scale * loss).backward()
    return li.detach().numpy(), float(loss.detach()), Xt.grad.numpy(), Wt.grad.numpy()


def test_full_softmax_matches_library_cross_entropy_fp64(orc):
    # the "tiny" configuration: C=10,000, D=128, B=64, s=30
    cfg = synth.CONFIGS["tiny"]
    W, X = synth.make_WX(cfg)
    y = synth.make_labels(cfg)
    full = orc.full_softmax_fwd_bwd(W, X, y, scale=cfg["scale"], grad_scale=1.0)
    li, loss, gX, gW = _torch_ce(W, X, np.arange(cfg["C"]), y, cfg["scale"], 1.0)
    assert np.allclose(full["loss_i"], li, rtol=1e-12, atol=1e-12)
    assert abs(full["loss"] - loss) <= 1e-12 * abs(loss)
    assert np.allclose(full["dX"], gX, rtol=1e-10, atol=1e-14)
    assert np.allclose(full["dW"], gW, rtol=1e-10, atol=1e-14)


def test_knn_softmax_matches_library_cross_entropy_on_active_columns(orc):
    cfg = synth.CONFIGS["tiny"]
    W, X = synth.make_WX(cfg)
    y = synth.make_labels(cfg)
    G = synth.graph_synthetic(7, cfg["C"], cfg["K"])
    active, A, tpos = orc.select_active(y, G, cfg["C"], cfg["M"])
    out = orc.knn_softmax_fwd_bwd(W, X, active[:A], tpos, scale=30.0, grad_scale=128.0)
    li, loss, gX, gW = _torch_ce(W, X, active[:A], tpos, 30.0, 128.0)
    assert np.allclose(out["loss_i"], li, rtol=1e-12, atol=1e-12)
    assert abs(out["loss"] - loss) <= 1e-12 * abs(loss)
    assert np.allclose(out["dX"], gX, rtol=1e-10, atol=1e-13)
    assert np.allclose(out["dWA"], gW, rtol=1e-10, atol=1e-13)


def test_closed_form_zero_features(orc):
    # X = 0 => all logits 0 => loss = ln A, P = 1/A, dZ = g (1/A - onehot), dX = s g (mean_a w_a - w_y)
    C, D, B, A = 500, 16, 4, 37
    W = synth.unit_rows(1, synth.TID_W, C, D)
    X = np.zeros((B, D), dtype=np.float32)
    active = np.sort(synth.class_permutation(1, C)[:A]).astype(np.int32)
    tpos = np.array([0, 5, 36, 5], dtype=np.int32)
    s, gs = 30.0, 3.0
    out = orc.knn_softmax_fwd_bwd(W, X, active, tpos, scale=s, grad_scale=gs, want_P=True)
    assert np.allclose(out["loss_i"], math.log(A), rtol=0, atol=1e-14)
    assert np.allclose(out["P"], 1.0 / A, rtol=0, atol=1e-15)
    WA = W[active].astype(np.float64)
    exp_dX = s * (gs / B) * (WA.mean(axis=0)[None, :] - WA[tpos])
    assert np.allclose(out["dX"], exp_dX, rtol=1e-12, atol=1e-15)
    assert np.allclose(out["dWA"], 0.0, atol=0)  # dWA = s dZ^T X with X = 0


def test_closed_form_single_active_class(orc):
    C, D, B = 50, 8, 3
    W, X, _ = _small_problem(C, D, B)
    out = orc.knn_softmax_fwd_bwd(W, X, np.array([17], dtype=np.int32), np.zeros(B, dtype=np.int32), 30.0, 1.0)
    assert (out["loss_i"] == 0).all() and out["loss"] == 0
    assert (out["dX"] == 0).all() and (out["dWA"] == 0).all()


def test_two_class_closed_form_and_no_overflow(orc):
    # x = w_0, w_1 = -w_0, s = 30: logits (30, -30); loss = log(1 + e^-60); P_1 = e^-60/(1+e^-60)
    D = 8
    w0 = np.zeros(D, dtype=np.float32)
    w0[2] = 1.0
    W = np.stack([w0, -w0])
    X = w0[None, :].copy()
    out = orc.knn_softmax_fwd_bwd(W, X, np.array([0, 1], dtype=np.int32), np.array([0], dtype=np.int32), 30.0, 1.0,
                                  want_P=True)
    e = math.exp(-60.0)
    assert out["loss"] == pytest.approx(math.log1p(e), rel=1e-12)
    assert out["P"][0, 1] == pytest.approx(e / (1 + e), rel=1e-12)
    # dX = s * (P0 w0 + P1 w1 - w0) = s * (-2 P1) w0
    assert out["dX"][0, 2] == pytest.approx(30.0 * (-2 * e / (1 + e)), rel=1e-10)
    # much larger spread still finite
    big = orc.knn_softmax_fwd_bwd(W, X, np.array([0, 1], dtype=np.int32), np.array([1], dtype=np.int32), 5000.0, 1.0)
    assert np.isfinite(big["loss"]) and big["loss"] == pytest.approx(10000.0, rel=1e-12)
    assert np.isfinite(big["dX"]).all() and np.isfinite(big["dWA"]).all()


def test_softmax_invariants(orc):
    cfg = synth.CONFIGS["tiny"]
    W, X = synth.make_WX(cfg)
    y = synth.make_labels(cfg)
    G = synth.graph_synthetic(11, cfg["C"], cfg["K"])
    active, A, tpos = orc.select_active(y, G, cfg["C"], cfg["M"])
    s, gs = 30.0, 1.0
    out = orc.knn_softmax_fwd_bwd(W, X, active[:A], tpos, s, gs, want_P=True)
    P = out["P"]
    assert np.abs(P.sum(axis=1) - 1.0).max() <= 1e-12
    assert (P >= 0).all()
    # sum_a dZ_ia = 0  =>  column sums of dWA vanish
    assert np.abs(out["dWA"].sum(axis=0)).max() <= 1e-13
    # dX_i = s g (sum_a P_ia w_a - w_{y_i})
    WA = W[active[:A]].astype(np.float64)
    exp_dX = s * (gs / cfg["B"]) * (P @ WA - WA[tpos])
    assert np.allclose(out["dX"], exp_dX, rtol=1e-10, atol=1e-14)
    # loss_i = -log P_{i, target}
    assert np.allclose(out["loss_i"], -np.log(P[np.arange(cfg["B"]), tpos]), rtol=1e-12, atol=1e-12)
    # grad_scale multiplies gradients only
    out2 = orc.knn_softmax_fwd_bwd(W, X, active[:A], tpos, s, 4.0)
    assert out2["loss"] == out["loss"]
    assert np.allclose(out2["dX"], 4.0 * out["dX"], rtol=1e-14, atol=0)
    assert np.allclose(out2["dWA"], 4.0 * out["dWA"], rtol=1e-14, atol=0)


def test_gradients_by_finite_differences(orc):
    # inputs on a 2^-12 grid and h a power of two, so that x +- h is exact in fp32; Richardson
    # extrapolation of the central difference removes the h^2 term
    C, D, B, A = 300, 16, 6, 40
    rng = np.random.default_rng(5)
    W = (np.round(rng.normal(0, 0.25, (C, D)) * 4096) / 4096).astype(np.float32)
    X = (np.round(rng.normal(0, 0.25, (B, D)) * 4096) / 4096).astype(np.float32)
    active = np.sort(rng.choice(C, A, replace=False)).astype(np.int32)
    tpos = rng.integers(0, A, B).astype(np.int32)
    s, gs = 8.0, 1.0
    base = orc.knn_softmax_fwd_bwd(W, X, active, tpos, s, gs)

    def loss_with(Wp, Xp):
        return orc.knn_softmax_fwd_bwd(Wp, Xp, active, tpos, s, gs)["loss"]

    def fd(which, r, d):
        vals = []
        for h in (2.0 ** -6, 2.0 ** -7):
            Wp, Wm_, Xp, Xm_ = W.copy(), W.copy(), X.copy(), X.copy()
            if which == "W":
                Wp[r, d] += h
                Wm_[r, d] -= h
            else:
                Xp[r, d] += h
                Xm_[r, d] -= h
            vals.append((loss_with(Wp, Xp) - loss_with(Wm_, Xm_)) / (2 * h))
        return (4 * vals[1] - vals[0]) / 3

    inactive = np.setdiff1d(np.arange(C), active)
    for _ in range(64):
        i, d = int(rng.integers(B)), int(rng.integers(D))
        assert fd("X", i, d) == pytest.approx(base["dX"][i, d], rel=2e-4, abs=1e-7)
        a, d = int(rng.integers(A)), int(rng.integers(D))
        assert fd("W", int(active[a]), d) == pytest.approx(base["dWA"][a, d], rel=2e-4, abs=1e-7)
        c, d = int(rng.choice(inactive)), int(rng.integers(D))
        assert fd("W", c, d) == 0.0  # classes outside the active set do not enter the loss


# --------------------------------------------------------------------------------------------
# Algorithm 1: selection
# --------------------------------------------------------------------------------------------
def _select_by_sets(labels, G, C, M):
    score = {}
    for y in labels.tolist():
        score[y] = 0
    for y in labels.tolist():
        for k, c in enumerate(G[y].tolist()):
            if c == -1:
                continue
            score[c] = min(score.get(c, 1 << 30), k + 1)
    classes = sorted(score)
    if len(classes) > M:
        classes = sorted(sorted(classes, key=lambda c: (score[c], c))[:M])
    pos = {c: a for a, c in enumerate(classes)}
    return np.array(classes, dtype=np.int32), np.array([pos[y] for y in labels.tolist()], dtype=np.int32)


@pytest.mark.parametrize("C,K,B,M,seed,empty", [(500, 8, 16, 400, 0, 0.0), (500, 8, 64, 100, 1, 0.0),
                                                (3000, 16, 128, 600, 2, 0.3), (64, 63, 8, 64, 3, 0.0),
                                                (200, 5, 200, 200, 4, 0.0)])
def test_selection_matches_set_based_definition(orc, C, K, B, M, seed, empty):
    G = synth.graph_synthetic(seed, C, K, locality=4, empty_frac=empty)
    y = synth.labels_uniform(seed, B, C)
    active, A, tpos = orc.select_active(y, G, C, M)
    exp_active, exp_tpos = _select_by_sets(y, G, C, M)
    assert A == len(exp_active) <= M
    assert (active[:A] == exp_active).all() and (active[A:] == -1).all()
    assert (tpos == exp_tpos).all()
    assert (active[tpos] == y).all()  # the label itself always survives (it heads its own list)
    assert (np.diff(active[:A]) > 0).all()


def test_selection_hand_built_cases(orc):
    C, K = 20, 3
    G = np.array([[(c + 1) % C, (c + 2) % C, (c + 3) % C] for c in range(C)], dtype=np.int32)
    # all labels equal: A = 1 + number of distinct neighbours
    a, A, t = orc.select_active(np.array([4, 4, 4], dtype=np.int32), G, C, 10)
    assert A == 4 and a[:4].tolist() == [4, 5, 6, 7] and t.tolist() == [0, 0, 0]
    # union of labels 4 and 6: {4,5,6,7,8,9}; scores: 4:0 5:1 6:0 7:1(from 6) 8:2 9:3
    y = np.array([4, 6], dtype=np.int32)
    a, A, t = orc.select_active(y, G, C, 6)        # M == |U|
    assert A == 6 and a[:6].tolist() == [4, 5, 6, 7, 8, 9]
    a, A, t = orc.select_active(y, G, C, 5)        # M == |U| - 1: the worst score (class 9, score 3) goes
    assert A == 5 and a[:5].tolist() == [4, 5, 6, 7, 8] and t.tolist() == [0, 2]
    # class 7 has rank 3 in list_4 but rank 1 in list_6: its score is 1, so it survives a cut to 4
    a, A, t = orc.select_active(y, G, C, 4)
    assert a[:4].tolist() == [4, 5, 6, 7]
    with pytest.raises(ValueError):
        orc.select_active(y, G, C, 3)              # a single label's list (K + 1 entries) must fit in M
    G2 = G.copy()
    G2[4] = [-1, 9, -1]                           # empty slots are skipped, ranks keep their column
    a, A, t = orc.select_active(np.array([4], dtype=np.int32), G2, C, 10)
    assert A == 2 and a[:2].tolist() == [4, 9]
    with pytest.raises(ValueError):
        orc.select_active(np.array([C], dtype=np.int32), G, C, 10)      # label out of range
    with pytest.raises(ValueError):
        orc.select_active(np.array([1, 2, 3], dtype=np.int32), G, C, 2)  # B > M


def test_selection_cut_tie_break_lowest_id(orc):
    C, K = 30, 2
    G = np.zeros((C, K), dtype=np.int32)
    G[:] = [[(c + 10) % C, (c + 20) % C] for c in range(C)]
    y = np.array([0, 1, 2], dtype=np.int32)
    # scores: 0,1,2 -> 0; 10,11,12 -> 1; 20,21,22 -> 2.  M = 5 keeps {0,1,2} + two lowest ids of score 1
    a, A, t = orc.select_active(y, G, C, 5)
    assert a[:A].tolist() == [0, 1, 2, 10, 11]
    a, A, t = orc.select_active(y, G, C, 7)
    assert a[:A].tolist() == [0, 1, 2, 10, 11, 12, 20]


# --------------------------------------------------------------------------------------------
# Section 3.2.2: neighbour search
# --------------------------------------------------------------------------------------------
def _graph_by_argsort(W64, K):
    S = W64 @ W64.T
    np.fill_diagonal(S, -np.inf)
    C = S.shape[0]
    ids = np.arange(C)
    out = np.empty((C, K), dtype=np.int32)
    for i in range(C):
        order = np.lexsort((ids, -S[i]))     # by similarity descending, then id ascending
        out[i] = order[:K]
    return out, S


def test_graph_matches_argsort_on_exact_integer_similarities(orc):
    # small integer entries: every inner product is an exact small integer in any summation order,
    # so there are masses of exact ties and the expected lists are unambiguous
    rng = np.random.default_rng(0)
    C, D, K = 400, 12, 9
    W = rng.integers(-2, 3, (C, D)).astype(np.float32)
    g, s = orc.graph_bruteforce(W, K)
    exp, S = _graph_by_argsort(W.astype(np.float64), K)
    assert (g == exp).all()
    assert (s == np.take_along_axis(S, exp.astype(np.int64), axis=1)).all()
    assert (np.diff(s, axis=1) <= 0).all()
    assert all(i not in g[i] for i in range(C))


def test_graph_one_hot_rows_tie_structure(orc):
    # rows are e_{i mod D}: similarity 1 inside a residue class, 0 otherwise => list of row i = lowest ids
    # of its residue class (without i), then the lowest ids overall that are not in the class
    C, D, K = 64, 8, 10
    W = np.zeros((C, D), dtype=np.float32)
    W[np.arange(C), np.arange(C) % D] = 1.0
    g, s = orc.graph_bruteforce(W, K)
    for i in range(C):
        same = [j for j in range(C) if j % D == i % D and j != i]
        other = [j for j in range(C) if j % D != i % D]
        assert g[i].tolist() == (same + other)[:K]
        assert s[i].tolist() == ([1.0] * len(same) + [0.0] * len(other))[:K]


def test_graph_duplicate_rows_and_random_rows(orc):
    C, D, K = 300, 24, 6
    W = synth.unit_rows(9, synth.TID_W, C, D)
    W[200] = W[17]                       # a twin: must come first in each other's list; self absent
    g, s = orc.graph_bruteforce(W, K)
    assert g[17, 0] == 200 and g[200, 0] == 17
    exp, S = _graph_by_argsort(W.astype(np.float64), K)
    assert (g == exp).all()              # random rows: no near-ties at fp64 resolution
    assert np.allclose(s, np.take_along_axis(S, exp.astype(np.int64), axis=1), rtol=0, atol=1e-15)
    # row subset API returns the same rows
    rows = np.array([5, 17, 299], dtype=np.int32)
    g2, s2 = orc.graph_bruteforce(W, K, rows)
    assert (g2 == g[rows]).all() and (s2 == s[rows]).all()
    # symmetry of the canonical similarity, bit-exact
    i, j = 17, int(g[17, 1])
    gi, si = orc.graph_bruteforce(W, C - 1, np.array([i, j], dtype=np.int32))
    assert si[0][gi[0].tolist().index(j)] == si[1][gi[1].tolist().index(i)]


# --------------------------------------------------------------------------------------------
# Section 3.1 step 6: local weight update
# --------------------------------------------------------------------------------------------
def test_apply_matches_dense_index_add(orc):
    C, D, n = 200, 16, 90
    rng = np.random.default_rng(2)
    W = synth.unit_rows(4, synth.TID_W, C, D)
    idx = rng.integers(0, 40, n).astype(np.int32)        # many repeats
    dW = synth.grad_rows(4, n, D)
    alpha = -0.37
    Wm, Wb = orc.apply_weight_grad(W, idx, dW, alpha)
    dense = np.zeros((C, D), dtype=np.float64)
    np.add.at(dense, idx, dW.astype(np.float64))
    exp = (W.astype(np.float64) + alpha * dense).astype(np.float32)
    assert (Wm == exp).all()
    touched = np.zeros(C, dtype=bool)
    touched[idx] = True
    assert (Wm[~touched] == W[~touched]).all()            # untouched rows bit-unchanged
    assert (Wb[~touched] == 0).all()
    assert (Wb[touched] == synth.bf16_bits(Wm[touched])).all()  # bf16 copy = RNE of the master


def test_bf16_rounding_to_nearest_even(orc):
    # values exactly between two bf16 neighbours must go to the even one
    W = np.array([[1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -1.0 - 2.0 ** -8]],
                 dtype=np.float32)
    Wm, Wb = orc.apply_weight_grad(W, np.array([0], dtype=np.int32), np.zeros((1, 4), dtype=np.float32), 1.0)
    got = synth.bf16_to_f32(Wb)[0].tolist()
    assert got == [1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -1.0]


# --------------------------------------------------------------------------------------------
# normalisation inside the layer (Section 3.2.1) and the update of un-normalised weights through it
# --------------------------------------------------------------------------------------------
def _raw_rows(seed, tid, n, D):
    """Rows of very different lengths (0.2 .. 5)."""
    V = synth.unit_rows(seed, tid, n, D).astype(np.float64)
    scale = 0.2 + 4.8 * ((np.arange(n) * 0.6180339887) % 1.0)
    return (V * scale[:, None]).astype(np.float32)


def test_normalize_rows_closed_forms(orc):
    V = _raw_rows(1, synth.TID_W, 50, 24)
    V[7] = 0.0
    Vh, Vb, inv = orc.normalize_rows(V)
    n = np.sqrt((V.astype(np.float64) ** 2).sum(axis=1))
    ok = n > 0
    assert np.allclose(inv[ok], 1.0 / n[ok], rtol=1e-6)
    assert np.allclose((Vh[ok].astype(np.float64) ** 2).sum(axis=1), 1.0, atol=1e-6)
    assert inv[7] == 0.0 and (Vh[7] == 0).all()
    # direction kept, length dropped: scaling a row changes nothing
    Vh2, _, _ = orc.normalize_rows(V * np.float32(4.0))    # power of two: the products are exact
    assert np.array_equal(Vh2, Vh)
    assert np.array_equal(Vb, synth.bf16_bits(Vh))
    # a 3-4-5 row
    Vh3, _, inv3 = orc.normalize_rows(np.array([[3.0, 4.0, 0.0]], dtype=np.float32))
    assert np.allclose(Vh3, [[0.6, 0.8, 0.0]], atol=1e-7) and abs(inv3[0] - 0.2) < 1e-8


def test_norm_backward_is_the_gradient_of_the_normalisation(orc):
    n, D = 12, 10
    V = _raw_rows(2, synth.TID_W, n, D)
    Cc = synth.unit_rows(5, synth.TID_X, n, D).astype(np.float64) * 3.0   # f(V) = sum_i <c_i, v_i / |v_i|>
    dV = orc.norm_backward(V, Cc)
    V64 = V.astype(np.float64)
    nrm = np.sqrt((V64 ** 2).sum(axis=1, keepdims=True))
    # closed form of the Jacobian-vector product: (c - v_hat <v_hat, c>) / |v|
    vh = V64 / nrm
    assert np.allclose(dV, (Cc - vh * (vh * Cc).sum(axis=1, keepdims=True)) / nrm, rtol=1e-12, atol=1e-14)
    # a gradient through a normalisation is orthogonal to the row, and scales inversely with its length
    assert np.abs((dV * V64).sum(axis=1)).max() < 1e-12
    dV2 = orc.norm_backward(V * np.float32(2.0), Cc)
    assert np.allclose(dV2, dV / 2.0, rtol=1e-12)
    # central differences in fp64 on f
    def f(Vx):
        return float((Cc * Vx / np.sqrt((Vx ** 2).sum(axis=1, keepdims=True))).sum())
    rng = np.random.default_rng(0)
    for _ in range(40):
        i, d = int(rng.integers(n)), int(rng.integers(D))
        h = 1e-6
        Vp, Vm = V64.copy(), V64.copy()
        Vp[i, d] += h
        Vm[i, d] -= h
        fd = (f(Vp) - f(Vm)) / (2 * h)
        assert abs(fd - dV[i, d]) <= 1e-7 * max(1.0, abs(dV[i, d]))
    # zero row: zero gradient
    V0 = V.copy()
    V0[3] = 0.0
    assert (orc.norm_backward(V0, Cc)[3] == 0).all()


def test_layer_with_normalisation_gradients_by_finite_differences(orc):
    """loss(W_raw, X_raw) = KNN-softmax loss on the normalised rows; the analytic gradient is the softmax
    oracle's gradient pushed through norm_backward."""
    C, D, B, K, M = 300, 12, 6, 4, 40
    Wr = _raw_rows(4, synth.TID_W, C, D)
    Xr = _raw_rows(4, synth.TID_X, B, D)
    y = synth.labels_uniform(4, B, C)
    G = synth.graph_synthetic(4, C, K, locality=2)
    active, A, tpos = orc.select_active(y, G, C, M)
    active = active[:A]
    s, gs = 8.0, 1.0

    def loss_of(W64, X64):
        Wh = W64 / np.sqrt((W64 ** 2).sum(axis=1, keepdims=True))
        Xh = X64 / np.sqrt((X64 ** 2).sum(axis=1, keepdims=True))
        Z = s * Xh @ Wh[active].T
        lse = np.log(np.exp(Z - Z.max(axis=1, keepdims=True)).sum(axis=1)) + Z.max(axis=1)
        return float((lse - Z[np.arange(B), tpos]).mean())

    Wh, _, _ = orc.normalize_rows(Wr, want_bf16=False)
    Xh, _, _ = orc.normalize_rows(Xr, want_bf16=False)
    out = orc.knn_softmax_fwd_bwd(Wh, Xh, active, tpos, s, gs)
    assert abs(out["loss"] - loss_of(Wr.astype(np.float64), Xr.astype(np.float64))) < 1e-6   # fp32 storage of the normalised rows
    dWr = orc.norm_backward(Wr[active], out["dWA"])
    dXr = orc.norm_backward(Xr, out["dX"])
    rng = np.random.default_rng(1)
    W64, X64 = Wr.astype(np.float64), Xr.astype(np.float64)
    for _ in range(30):
        a, d = int(rng.integers(A)), int(rng.integers(D))
        h = 1e-5
        Wp, Wm_ = W64.copy(), W64.copy()
        Wp[active[a], d] += h
        Wm_[active[a], d] -= h
        fd = (loss_of(Wp, X64) - loss_of(Wm_, X64)) / (2 * h)
        assert abs(fd - dWr[a, d]) <= 2e-5 * max(abs(dWr[a, d]), 1e-3), (fd, dWr[a, d])
    for _ in range(30):
        i, d = int(rng.integers(B)), int(rng.integers(D))
        h = 1e-5
        Xp, Xm = X64.copy(), X64.copy()
        Xp[i, d] += h
        Xm[i, d] -= h
        fd = (loss_of(W64, Xp) - loss_of(W64, Xm)) / (2 * h)
        assert abs(fd - dXr[i, d]) <= 2e-5 * max(abs(dXr[i, d]), 1e-3), (fd, dXr[i, d])


def test_apply_weight_grad_normalized_against_numpy(orc):
    C, D, n = 40, 16, 25
    W = _raw_rows(6, synth.TID_W, C, D)
    rng = np.random.default_rng(2)
    idx = rng.integers(0, C // 2, n).astype(np.int32)          # repeats; the upper half stays untouched
    dWh = synth.grad_rows(6, n, D).astype(np.float32)
    alpha = -0.3
    Wm, Wb, inv = orc.apply_weight_grad_normalized(W, idx, dWh, alpha)
    W64 = W.astype(np.float64)
    exp = W64.copy()
    for c in np.unique(idx):
        g = dWh[idx == c].astype(np.float64).sum(axis=0)
        nrm = np.sqrt((W64[c] ** 2).sum())
        wh = W64[c] / nrm
        exp[c] = W64[c] + alpha * (g - wh * (wh @ g)) / nrm
    assert np.allclose(Wm, exp, rtol=0, atol=2.0 ** -23 * np.abs(exp).max())
    touched = np.unique(idx)
    untouched = np.setdiff1d(np.arange(C), touched)
    assert np.array_equal(Wm[untouched], W[untouched]) and (Wb[untouched] == 0).all() and (inv[untouched] == 0).all()
    n2 = np.sqrt((Wm[touched].astype(np.float64) ** 2).sum(axis=1))
    assert np.allclose(inv[touched], 1.0 / n2, rtol=1e-6)
    assert np.array_equal(Wb[touched], synth.bf16_bits((Wm[touched].astype(np.float64) / n2[:, None]).astype(np.float32)))
    # first-order property of a step through a normalisation: the length of a row changes only in second order
    n1 = np.sqrt((W64[touched] ** 2).sum(axis=1))
    step = np.sqrt(((Wm[touched] - W[touched]).astype(np.float64) ** 2).sum(axis=1))
    assert np.all(np.abs(n2 - n1) <= step ** 2 / n1 + 1e-6)


def test_apply_weight_grad_normalized_is_a_gradient_step_of_a_loss_of_the_normalised_rows(orc):
    """Independent of the projection formula: take any scalar loss L(W) = f(W_hat) of the normalised rows, hand the
    update the gradient of f with respect to W_hat, and the change of W must be alpha times the gradient of L with
    respect to W itself -- which central differences of L (normalisation written out in numpy, fp64) give without
    any formula for the Jacobian.  f is a cubic, so that its gradient depends on the point."""
    C, D = 12, 10
    W = _raw_rows(8, synth.TID_W, C, D)
    W64 = W.astype(np.float64)
    Q = synth.normal(8, synth.TID_MISC, 0, C * D).reshape(C, D)
    R = synth.normal(9, synth.TID_MISC, 0, C * D).reshape(C, D)

    def hat(V):
        return V / np.sqrt((V * V).sum(axis=1, keepdims=True))

    def loss(V):                                   # f(V_hat) = sum Q * V_hat + sum R * V_hat^3
        H = hat(V)
        return float((Q * H).sum() + (R * H ** 3).sum())

    H0 = hat(W64)
    grad_f = (Q + 3.0 * R * H0 ** 2).astype(np.float32)      # df/dW_hat at the starting point (what the layer passes on)
    idx = np.array([1, 4, 7, 9, 11], dtype=np.int32)
    alpha = -0.125
    Wm, _, _ = orc.apply_weight_grad_normalized(W, idx, grad_f[idx], alpha)
    h = 1e-6
    for c in idx:
        fd = np.empty(D)
        for d in range(D):
            Vp, Vn = W64.copy(), W64.copy()
            Vp[c, d] += h
            Vn[c, d] -= h
            fd[d] = (loss(Vp) - loss(Vn)) / (2 * h)
        step = Wm[c].astype(np.float64) - W64[c]
        assert np.abs(step - alpha * fd).max() <= 1e-6 * np.abs(alpha * fd).max() + 2.0 ** -23 * np.abs(W64[c]).max()
    rest = np.setdiff1d(np.arange(C), idx)
    assert np.array_equal(Wm[rest], W[rest])


def test_apply_weight_grad_normalized_equals_the_two_pinned_steps_composed(orc):
    """Projection through the normalisation (orc_norm_backward, pinned by finite differences) followed by the plain
    update (orc_apply_weight_grad, pinned against numpy's add.at): the same master rows up to the fp32 rounding of the
    projected gradient that the composed version hands over; repeated indices included (the projection is linear)."""
    C, D, n = 60, 24, 40
    W = _raw_rows(10, synth.TID_W, C, D)
    rng = np.random.default_rng(4)
    idx = rng.integers(0, C // 2, n).astype(np.int32)
    dWh = synth.grad_rows(10, n, D).astype(np.float32)
    alpha = 0.2
    Wm, Wb, inv = orc.apply_weight_grad_normalized(W, idx, dWh, alpha)
    dW = orc.norm_backward(W[idx], dWh.astype(np.float64))                 # row p: projected with the row of class idx[p]
    Wc, _ = orc.apply_weight_grad(W, idx, dW.astype(np.float32), alpha, want_bf16=False)
    mult = np.bincount(idx, minlength=C).max()
    tol = 2.0 ** -23 * np.abs(Wc).max() + mult * 2.0 ** -24 * abs(alpha) * np.abs(dW).max()
    assert np.abs(Wm.astype(np.float64) - Wc).max() <= tol
    # the refreshed copies describe the stored rows (normalize_rows has its own closed-form pins)
    touched = np.unique(idx)
    _, eb, einv = orc.normalize_rows(Wm[touched])
    assert np.array_equal(Wb[touched], eb) and np.array_equal(inv[touched], einv)


# ------------------------------------------------------------------------------------------------
# compressed graph of one node, selection on it, random fill-up (Section 3.2.3, Algorithm 1)
# ------------------------------------------------------------------------------------------------
def test_graph_compress_by_brute_force_and_partition(orc):
    Cg, K = 37, 5
    G = synth.graph_synthetic(3, Cg, K, locality=8, empty_frac=0.2)
    bounds = [0, 10, 11, 30, 37]                                  # four nodes of unequal size (one owns one class)
    seen = [[] for _ in range(Cg)]
    for c0, c1 in zip(bounds[:-1], bounds[1:]):
        counts, offsets, flat = orc.graph_compress(G, c0, c1 - c0)
        assert offsets[0] == 0 and np.array_equal(offsets[1:], np.cumsum(counts)) and len(flat) == offsets[-1]
        for g in range(Cg):
            want = [int(c) - c0 for c in G[g] if c0 <= c < c1]   # the node's part of the list, order kept
            assert flat[offsets[g]:offsets[g + 1]].tolist() == want
            seen[g] += [c + c0 for c in want]
    for g in range(Cg):                                           # the nodes' parts partition every list
        assert sorted(seen[g]) == sorted(int(c) for c in G[g] if c >= 0)


def test_selection_on_compressed_graph_hand_worked_case(orc):
    # eight classes, the node owns 4..7; K = 3
    G = np.array([[5, 1, 6], [4, 7, 2], [6, 5, 4], [0, 1, 2], [0, 1, 2], [0, 1, 2], [7, 0, 5], [0, 1, 2]], dtype=np.int32)
    counts, offsets, flat = orc.graph_compress(G, 4, 4)
    assert counts.tolist() == [2, 2, 3, 0, 0, 0, 2, 0]
    assert flat.tolist() == [1, 2, 0, 3, 2, 1, 0, 3, 1]
    labels = np.array([0, 1, 6], dtype=np.int32)
    # sample 0 (class 0, another node's): local 1 at position 1, local 2 at 2; sample 1 (class 1): local 0 at 1,
    # local 3 at 2; sample 2 (class 6 = local 2, owned): itself at 0, local 3 at 1, local 1 at 2
    # => scores: local 0: 1, local 1: 1, local 2: 0, local 3: 1
    a, n, nf, t = orc.select_active_csr(labels, counts, offsets, flat, 4, 4, 4)
    assert (a.tolist(), n, nf, t.tolist()) == ([0, 1, 2, 3], 4, 4, [-1, -1, 2])
    a, n, nf, t = orc.select_active_csr(labels, counts, offsets, flat, 4, 4, 3)
    assert (a.tolist(), n, nf, t.tolist()) == ([0, 1, 2], 3, 3, [-1, -1, 2])    # score 0 first, then the lowest ids at score 1
    # a node that owns none of the labels and nothing in their lists finds nothing
    c2, o2, f2 = orc.graph_compress(G, 3, 1)
    a, n, nf, t = orc.select_active_csr(labels, c2, o2, f2, 3, 1, 4)
    assert (a.tolist(), n, nf, t.tolist()) == ([-1, -1, -1, -1], 0, 0, [-1, -1, -1])


@pytest.mark.parametrize("Cg,K,B,M,seed", [(500, 6, 40, 400, 0), (500, 6, 40, 60, 1), (2000, 12, 100, 300, 2)])
def test_selection_on_one_node_owning_everything_equals_the_dense_selection(orc, Cg, K, B, M, seed):
    G = synth.graph_synthetic(seed, Cg, K, locality=16)          # no empty slots: positions survive the compression
    labels = synth.labels_uniform(seed, B, Cg)
    counts, offsets, flat = orc.graph_compress(G, 0, Cg)
    assert (counts == K).all() and np.array_equal(flat.reshape(Cg, K), G)
    a0, n0, t0 = orc.select_active(labels, G, Cg, M)
    a1, n1, nf, t1 = orc.select_active_csr(labels, counts, offsets, flat, 0, Cg, M)
    assert n0 == n1 == nf and np.array_equal(a0, a1) and np.array_equal(t0, t1)


def test_selection_over_all_nodes_reassembles_the_dense_selection(orc):
    Cg, K, B, P = 3000, 10, 64, 4
    G = synth.graph_synthetic(5, Cg, K, locality=32, empty_frac=0.1)
    labels = synth.labels_uniform(5, B, Cg)
    M = 2000                                                      # no cut anywhere
    a0, n0, t0 = orc.select_active(labels, G, Cg, M)
    union, owners = [], np.zeros(B, dtype=int)
    for p in range(P):
        c0, C_loc = p * Cg // P, (p + 1) * Cg // P - p * Cg // P
        counts, offsets, flat = orc.graph_compress(G, c0, C_loc)
        a, n, nf, t = orc.select_active_csr(labels, counts, offsets, flat, c0, C_loc, M)
        assert n == nf and (a[n:] == -1).all() and (np.diff(a[:n]) > 0).all()
        union += (a[:n] + c0).tolist()
        own = (labels >= c0) & (labels < c0 + C_loc)
        assert (t[~own] == -1).all() and np.array_equal(a[t[own]] + c0, labels[own])
        owners += own
    assert (owners == 1).all() and union == a0[:n0].tolist()      # ascending node by node = ascending overall


def test_fill_up_order_is_one_to_one(orc):
    for C_loc, seed in [(1, 0), (2, 1), (3, 2), (64, 3), (65, 4), (1000, 5), (390625, 6), (390625, 7 << 40)]:
        b = max(1, int(np.ceil(np.log2(C_loc))))
        d = orc.pad_draws(C_loc, seed, 1 << b)
        assert d.max() == (1 << b) - 1 and len(np.unique(d)) == 1 << b
    a, b_ = orc.pad_draws(390625, 6, 4096), orc.pad_draws(390625, 7 << 40, 4096)
    assert len(np.intersect1d(a, b_)) < 200                       # another seed, another order


def test_fill_up_takes_the_first_draws_not_yet_chosen(orc):
    Cg, K, B, c0, C_loc = 4000, 8, 50, 1000, 1500
    G = synth.graph_synthetic(8, Cg, K, locality=16)
    labels = synth.labels_uniform(8, B, Cg)
    counts, offsets, flat = orc.graph_compress(G, c0, C_loc)
    for M, seed in [(256, 11), (1500, 12), (3000, 13)]:
        a0, n0, nf0, t0 = orc.select_active_csr(labels, counts, offsets, flat, c0, C_loc, M)
        a1, n1, nf1, t1 = orc.select_active_csr(labels, counts, offsets, flat, c0, C_loc, M, pad=True, seed=seed)
        assert nf1 == nf0 == n0 and n1 == min(M, C_loc) and (np.diff(a1[:n1]) > 0).all()
        found, final = set(a0[:n0].tolist()), set(a1[:n1].tolist())
        assert found <= final
        draws = [int(c) for c in orc.pad_draws(C_loc, seed, 4096) if c < C_loc and int(c) not in found]
        assert final - found == set(draws[:n1 - n0])
        own = (labels >= c0) & (labels < c0 + C_loc)
        assert (t1[~own] == -1).all() and np.array_equal(a1[t1[own]] + c0, labels[own])
    # nothing to fill when the cut bites
    a2, n2, nf2, _ = orc.select_active_csr(labels, counts, offsets, flat, c0, C_loc, 60, pad=True, seed=1)
    a3, n3, _, _ = orc.select_active_csr(labels, counts, offsets, flat, c0, C_loc, 60)
    assert n2 == nf2 == 60 and np.array_equal(a2, a3)


def test_fill_up_is_uniform_over_the_classes_not_chosen(orc):
    # 40 classes, 8 found by the lists; 8 more drawn from the other 32 under 4,000 seeds: each with probability 1/4
    Cg = C_loc = 40
    G = ((np.arange(Cg)[:, None] + 1 + np.arange(3)[None, :]) % Cg).astype(np.int32)
    labels = np.array([0, 20], dtype=np.int32)                    # finds 0..3 and 20..23
    counts, offsets, flat = orc.graph_compress(G, 0, C_loc)
    hits = np.zeros(C_loc)
    n_seeds = 4000
    for seed in range(n_seeds):
        a, n, nf, _ = orc.select_active_csr(labels, counts, offsets, flat, 0, C_loc, 16, pad=True, seed=seed * 2654435761 + 17)
        assert n == 16 and nf == 8
        hits[a[:n]] += 1
    found = [0, 1, 2, 3, 20, 21, 22, 23]
    assert (hits[found] == n_seeds).all()
    rest = np.delete(hits, found)
    sigma = np.sqrt(n_seeds * 0.25 * 0.75)
    assert np.abs(rest - n_seeds * 0.25).max() < 5 * sigma
    chi2 = ((rest - n_seeds * 0.25) ** 2 / (n_seeds * 0.25 * 0.75)).sum()
    assert chi2 < 32 + 6 * np.sqrt(2 * 32)


# ------------------------------------------------------------------------------------------------
# one hop of the distributed graph build (Section 3.2.2): merging a visiting shard into the lists
# ------------------------------------------------------------------------------------------------
def _empty_lists(n, K):
    return np.full((n, K), -1, dtype=np.int32), np.full((n, K), -np.inf)


@pytest.mark.parametrize("bounds,order", [([0, 150, 300], [0, 1]), ([0, 150, 300], [1, 0]), ([0, 40, 41, 170, 300], [2, 0, 3, 1]),
                                          ([0, 300], [0])])
def test_graph_hops_over_all_shards_give_the_brute_force_graph(orc, bounds, order):
    C, D, K = 300, 32, 7
    W = synth.clustered_rows(4, C, D, n_centres=20, noise=0.4)
    W[17] = W[3]                                                  # duplicate rows: ties decided by the id
    W[250] = W[3]
    G, S = orc.graph_bruteforce(W, K)
    shards = list(zip(bounds[:-1], bounds[1:]))
    for a, b in shards:                                           # every node in turn
        g, s = _empty_lists(b - a, K)
        for v in order:
            va, vb = shards[v]
            g, s = orc.graph_update(W[a:b], W[va:vb], a, va, g, s)
        assert np.array_equal(g, G[a:b]) and np.array_equal(s, S[a:b])
        g2, s2 = orc.graph_update(W[a:b], W[shards[0][0]:shards[0][1]], a, shards[0][0], g, s)   # a shard seen twice
        assert np.array_equal(g2, g) and np.array_equal(s2, s)


def test_graph_hop_hand_worked_case(orc):
    # node owns ids 10, 11 (rows e0, e1); the visiting shard holds ids 4..6: e0, e1, (e0 + e1)
    e = np.eye(4, dtype=np.float32)
    W_local = np.stack([e[0], e[1]])
    W_visit = np.stack([e[0], e[1], e[0] + e[1]])
    g, s = _empty_lists(2, 2)
    g, s = orc.graph_update(W_local, W_visit, 10, 4, g, s)
    assert g.tolist() == [[4, 6], [5, 6]] and s.tolist() == [[1.0, 1.0], [1.0, 1.0]]         # ties: lower id first
    # a second shard with ids 0..1: 2*e0 and e1 -- beats everything for row 10, ties for row 11
    g, s = orc.graph_update(W_local, np.stack([2 * e[0], e[1]]), 10, 0, g, s)
    assert g.tolist() == [[0, 4], [1, 5]] and s.tolist() == [[2.0, 1.0], [1.0, 1.0]]
    # the node's own shard: the row itself is skipped, the other row has similarity 0 and does not make the list
    g, s = orc.graph_update(W_local, W_local, 10, 10, g, s)
    assert g.tolist() == [[0, 4], [1, 5]]
    # fewer candidates than K: empty slots stay -1 / -inf
    g, s = orc.graph_update(W_local, W_local[:1], 10, 10, *_empty_lists(2, 2))
    assert g.tolist() == [[-1, -1], [10, -1]] and s[0].tolist() == [-np.inf, -np.inf] and s[1].tolist() == [0.0, -np.inf]


# ------------------------------------------------------------------------------------------------
# the softmax split over nodes (Section 3.1 steps 3-5)
# ------------------------------------------------------------------------------------------------
def test_softmax_split_over_nodes_equals_the_softmax_on_one_gpu(orc):
    C, D, B, K, s, gs, P = 600, 24, 20, 6, 12.0, 64.0, 3
    W = synth.unit_rows(31, synth.TID_W, C, D)
    y = synth.labels_uniform(31, B, C)
    X = synth.features_near_labels(31, W, y, sigma=1.0)
    G = synth.graph_synthetic(31, C, K, locality=16)
    active, A, tpos = orc.select_active(y, G, C, 512)
    ref = orc.knn_softmax_fwd_bwd(W, X, active[:A], tpos, s, gs)
    bounds = [0, 150, 420, 600]
    nodes = []
    for c0, c1 in zip(bounds[:-1], bounds[1:]):
        counts, offsets, flat = orc.graph_compress(G, c0, c1 - c0)
        a, n, _, t = orc.select_active_csr(y, counts, offsets, flat, c0, c1 - c0, 512)
        nodes.append((c0, c1, a[:n], t))
    stats = [orc.softmax_node_stats(W[c0:c1], X, a, t, s) for c0, c1, a, t in nodes]
    Mg, Sg, Tg = orc.combine_node_stats(stats)
    assert np.allclose(Mg + np.log(Sg), ref["lse"], rtol=0, atol=1e-12)
    dX = np.zeros((B, D))
    dW_rows = {}
    for (c0, c1, a, t), (m, l, tz) in zip(nodes, stats):
        out = orc.softmax_node_bwd(W[c0:c1], X, a, t, s, gs, Mg, Sg, Tg)
        assert np.allclose(out["loss_i"], ref["loss_i"], rtol=0, atol=1e-11) and abs(out["loss"] - ref["loss"]) < 1e-12
        dX += out["dX"]
        for r, c in enumerate(a):
            dW_rows[int(c) + c0] = out["dWA"][r]
        # another pair (m, l) for the same sums gives the same statistics after combining
        shifted = [(mm - 3.0, ll * np.exp(3.0), tt) if k == 0 else (mm, ll, tt) for k, (mm, ll, tt) in enumerate(stats)]
        M2, S2, _ = orc.combine_node_stats(shifted)
        assert np.allclose(M2 + np.log(S2), Mg + np.log(Sg), rtol=0, atol=1e-12)
    assert np.allclose(dX, ref["dX"], rtol=0, atol=1e-13 * gs)
    assert sorted(dW_rows) == active[:A].tolist()
    assert np.allclose(np.stack([dW_rows[int(c)] for c in active[:A]]), ref["dWA"], rtol=0, atol=1e-13 * gs)
    # every sample has its target on exactly one node, and that node reports the target's logit
    owners = np.sum([(t >= 0).astype(int) for _, _, _, t in nodes], axis=0)
    assert (owners == 1).all()
    Z = s * X.astype(np.float64) @ W.astype(np.float64).T
    assert np.allclose(Tg, Z[np.arange(B), y], rtol=0, atol=1e-12)


def test_softmax_node_with_a_single_column_closed_form(orc):
    # one node holding one class, one sample whose class lives elsewhere: m = z, l = 1, t = 0; with the other node's
    # statistics (M, S, T) the gradient of the only logit is g * exp(z - M) / S
    W = np.array([[0.6, 0.8]], dtype=np.float32)
    X = np.array([[1.0, 0.0]], dtype=np.float32)
    m, l, t = orc.softmax_node_stats(W, X, np.array([0], dtype=np.int32), np.array([-1], dtype=np.int32), 10.0)
    assert abs(m[0] - 6.0) < 1e-6 and l[0] == 1.0 and t[0] == 0.0
    out = orc.softmax_node_bwd(W, X, np.array([0], dtype=np.int32), np.array([-1], dtype=np.int32), 10.0, 2.0,
                               np.array([8.0]), np.array([1.5]), np.array([7.0]))
    dz = 2.0 * np.exp(m[0] - 8.0) / 1.5
    assert abs(out["loss"] - (8.0 + np.log(1.5) - 7.0)) < 1e-12
    assert np.allclose(out["dX"][0], 10.0 * dz * W[0].astype(np.float64)) and np.allclose(out["dWA"][0], 10.0 * dz * X[0])
