"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.
Integer outputs (active list, positions, neighbour lists) must be bit-exact; floating point within
loss rel. error <= 1e-3 and dX / dW relative Frobenius error <= 2e-2 (bf16 operands, fp32 accumulate)."""
import numpy as np
import pytest
import torch

import synth
from gradcheck import GRAD_RTOL, check_rows, check_step_grads, grad_floors

pytestmark = pytest.mark.gpu

LOSS_RTOL = 1e-3
SENTINEL = -12345.0


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
    den = np.linalg.norm(b)
    return np.linalg.norm(a - b) / den if den > 0 else np.linalg.norm(a - b)


def run_and_compare(ks, orc, W, X, y, G, C, M, scale=30.0, grad_scale=1.0, tag="", modes=(False, True)):
    """W, X fp32 arrays on the bf16 grid.  Runs both sides and checks every output, without and with the
    unit-rows promise (the one-sweep softmax; the same results are required).  Returns the last mode's output."""
    active, A, tpos = orc.select_active(y, G, C, M)
    ref = orc.knn_softmax_fwd_bwd(W, X, active[:A], tpos, scale, grad_scale)
    for unit_rows in modes:
        out = _run_and_compare_one(ks, W, X, y, G, C, M, scale, grad_scale, tag, unit_rows, active, A, tpos, ref)
    return out, ref, A


def _run_and_compare_one(ks, W, X, y, G, C, M, scale, grad_scale, tag, unit_rows, active, A, tpos, ref):
    print(f"[case] {tag} C={C} D={W.shape[1]} B={X.shape[0]} K={G.shape[1]} M={M} unit_rows={unit_rows}", flush=True)
    B, D = X.shape
    # the gradient buffers start from a sentinel: every row that must be written is, and no row beyond is
    bufs = dict(active_idx=torch.empty(M, dtype=torch.int32, device="cuda"),
                n_active=torch.empty(1, dtype=torch.int32, device="cuda"),
                target_pos=torch.empty(B, dtype=torch.int32, device="cuda"),
                loss_per_sample=torch.empty(B, dtype=torch.float32, device="cuda"),
                loss_mean=torch.empty(1, dtype=torch.float32, device="cuda"),
                dX=torch.full((B, D), SENTINEL, dtype=torch.float32, device="cuda"),
                dW_active=torch.full((M, D), SENTINEL, dtype=torch.float32, device="cuda"))
    out = ks.knn_softmax_fwd_bwd(dev(W, torch.bfloat16), dev(X, torch.bfloat16), dev(y), dev(G), M, scale, grad_scale,
                                 out=bufs, unit_rows=unit_rows)
    torch.cuda.synchronize()
    assert int(out["dev_status"].item()) == 0
    assert int(out["n_active"].item()) == A
    assert (out["active_idx"].cpu().numpy() == active).all()
    assert (out["target_pos"].cpu().numpy() == tpos).all()
    li = out["loss_per_sample"].cpu().numpy()
    assert np.abs(li - ref["loss_i"]).max() <= LOSS_RTOL * max(1.0, np.abs(ref["loss_i"]).max())
    loss = float(out["loss_mean"].item())
    assert abs(loss - ref["loss"]) <= LOSS_RTOL * abs(ref["loss"]), (loss, ref["loss"])
    print(f"        A={A} loss={loss:.6f} ref={ref['loss']:.6f}", flush=True)
    # every sample's row of dX and every active class's row of dW_A against the oracle's
    check_step_grads(out["dX"].cpu().numpy(), out["dW_active"][:A].cpu().numpy(), ref, W[active[:A]], X, tpos, scale,
                     grad_scale, tag=tag)
    assert bool((out["dW_active"][A:] == SENTINEL).all()), "rows beyond n_active were written"
    return out


# ------------------------------------------------------------------------------------------------
# selection alone
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("C,K,B,M,seed,empty", [
    (500, 8, 16, 400, 0, 0.0),          # no cut
    (500, 8, 64, 100, 1, 0.0),          # cut bites
    (3000, 16, 128, 600, 2, 0.3),       # empty slots
    (64, 63, 8, 64, 3, 0.0),            # lists span all classes
    (200, 5, 200, 200, 4, 0.0),         # B == M
    (100_000, 16, 256, 4_096, 0, 0.0),  # the "small" configuration: cut bites
    (390_625, 32, 1_024, 32_768, 0, 0.0),
    (390_625, 32, 1_024, 20_000, 1, 0.1),   # single-workgroup path, cut bites
    (393_217, 16, 512, 4_000, 2, 0.0),      # just above the single-workgroup limit: table path, cut bites
    (1_000_000, 64, 2_048, 131_072, 0, 0.0),
    (5000, 2500, 4, 3000, 5, 0.0),      # more list positions than the LDS histogram holds
])
def test_select_matches_oracle(ks, orc, C, K, B, M, seed, empty):
    G = synth.graph_synthetic(seed, C, K, locality=4, empty_frac=empty)
    y = synth.labels_uniform(seed, B, C)
    a, n, t, st = ks.knn_select_active(dev(y), dev(G), C, M)
    torch.cuda.synchronize()
    ea, eA, et = orc.select_active(y, G, C, M)
    assert int(st.item()) == 0
    assert int(n.item()) == eA
    assert (a.cpu().numpy() == ea).all()
    assert (t.cpu().numpy() == et).all()


def test_select_without_graph_and_flags(ks, orc):
    y = np.array([5, 3, 5, 9], dtype=np.int32)
    a, n, t, st = ks.knn_select_active(dev(y), None, 10, 6)
    assert int(n.item()) == 3 and a.cpu().numpy().tolist() == [3, 5, 9, -1, -1, -1]
    assert t.cpu().numpy().tolist() == [1, 0, 1, 2]
    # out-of-range label / neighbour id: flagged, no crash
    G = synth.graph_synthetic(0, 50, 4)
    G[7, 2] = 50
    a, n, t, st = ks.knn_select_active(dev(np.array([7, 60], dtype=np.int32)), dev(G), 50, 20)
    torch.cuda.synchronize()
    assert int(st.item()) == (ks.KS_DEV_BAD_LABEL | ks.KS_DEV_BAD_GRAPH_ID)


# ------------------------------------------------------------------------------------------------
# forward + backward
# ------------------------------------------------------------------------------------------------
def test_fwd_bwd_tiny_config(ks, orc):
    cfg = synth.CONFIGS["tiny"]
    W = synth.bf16_round(synth.unit_rows(0, synth.TID_W, cfg["C"], cfg["D"]))
    X = synth.bf16_round(synth.unit_rows(0, synth.TID_X, cfg["B"], cfg["D"]))
    y = synth.make_labels(cfg)
    G, _ = orc.graph_bruteforce(W, cfg["K"])         # true KNN graph of W, all rows
    run_and_compare(ks, orc, W, X, y, G, cfg["C"], cfg["M"], tag="tiny")


def test_fwd_bwd_small_config_cut_bites(ks, orc):
    cfg = synth.CONFIGS["small"]
    W, X = synth.make_WX(cfg)
    y = synth.make_labels(cfg)
    G = synth.graph_synthetic(0, cfg["C"], cfg["K"], locality=2)
    rows = np.unique(y)
    G[rows], _ = orc.graph_bruteforce(W, cfg["K"], rows)   # true neighbours for the rows selection reads
    out, ref, A = run_and_compare(ks, orc, W, X, y, G, cfg["C"], cfg["M"], tag="small")
    assert A == cfg["M"]                                   # about 4,250 distinct candidates > M = 4,096


@pytest.mark.parametrize("C,D,B,K,M,seed", [(3000, 96, 50, 7, 333, 1), (777, 32, 1, 4, 5, 2), (5000, 160, 130, 9, 1111, 3),
                                             (2000, 64, 257, 3, 1000, 4)])
def test_fwd_bwd_ragged_shapes(ks, orc, C, D, B, K, M, seed):
    W = synth.unit_rows(seed, synth.TID_W, C, D, bf16=True)
    X = synth.unit_rows(seed, synth.TID_X, B, D, bf16=True)
    y = synth.labels_uniform(seed, B, C)
    G = synth.graph_synthetic(seed, C, K, locality=4)
    run_and_compare(ks, orc, W, X, y, G, C, M, grad_scale=128.0, tag="ragged")


def test_fwd_bwd_peaky_softmax_and_clustered_weights(ks, orc):
    # features close to their class weight (target logit near the scale), clustered weights (many near-equal logits)
    C, D, B, K, M = 20_000, 256, 192, 16, 2_048
    W = synth.clustered_rows(3, C, D, n_centres=512, bf16=True)
    y = synth.labels_zipf(3, B, C)
    X = synth.features_near_labels(3, W, y, sigma=0.4, bf16=True)
    rows = np.unique(y)
    G = synth.graph_synthetic(3, C, K)
    G[rows], _ = orc.graph_bruteforce(W, K, rows)
    out, ref, A = run_and_compare(ks, orc, W, X, y, G, C, M, tag="peaky")
    # the per-sample losses span orders of magnitude here; check them relatively where they are not tiny
    li = out["loss_per_sample"].cpu().numpy()
    big = ref["loss_i"] > 1e-2
    assert (np.abs(li[big] - ref["loss_i"][big]) <= 5e-3 * ref["loss_i"][big] + 1e-3).all()


@pytest.mark.parametrize("D,noise,sigma", [(128, 0.5, 0.2), (256, 0.5, 0.2), (512, 0.6, 0.3)])
def test_one_sweep_loss_of_confident_samples_is_accurate_sample_by_sample(ks, orc, D, noise, sigma):
    """Confident samples (the own class takes nearly all of the probability) among classes that come in pairs of
    near twins, so that a single competitor holds nearly all of what is left: the one-sweep mode must not let the
    bf16 rounding of that competitor's stored exponential (2^-9, above the 1e-3 bound) into the loss.  Checked
    relatively, sample by sample."""
    C, B, K, M = 12_000, 256, 16, 2_048
    W = synth.clustered_rows(11, C, D, n_centres=C // 2, noise=noise, bf16=True)
    y = synth.labels_zipf(11, B, C)
    X = synth.features_near_labels(11, W, y, sigma=sigma, bf16=True)
    rows = np.unique(y)
    G = synth.graph_synthetic(11, C, K)
    G[rows], _ = orc.graph_bruteforce(W, K, rows)
    active, A, tpos = orc.select_active(y, G, C, M)
    ref = orc.knn_softmax_fwd_bwd(W, X, active[:A], tpos, 30.0, 1.0)
    out = ks.knn_softmax_fwd_bwd(dev(W, torch.bfloat16), dev(X, torch.bfloat16), dev(y), dev(G), M, 30.0, 1.0, unit_rows=True)
    torch.cuda.synchronize()
    assert int(out["dev_status"].item()) == 0
    li, rl = out["loss_per_sample"].cpu().numpy().astype(np.float64), ref["loss_i"]
    err = np.abs(li - rl) / (rl + 1e-6)
    print(f"        D={D}: losses from {rl.min():.2e} to {rl.max():.2e}, median {np.median(rl):.2e}; "
          f"worst relative error {err.max():.2e}", flush=True)
    assert np.median(rl) < 0.05, "the case is meant to be confident"
    assert err.max() <= 5e-4


def test_knn_equals_full_softmax_when_lists_span_all_classes(ks, orc):
    C, D, B = 4_000, 128, 96
    W = synth.unit_rows(8, synth.TID_W, C, D, bf16=True)
    X = synth.unit_rows(8, synth.TID_X, B, D, bf16=True)
    y = synth.labels_uniform(8, B, C)
    G = synth.graph_all_others(C)
    out, ref, A = run_and_compare(ks, orc, W, X, y, G, C, C, tag="K=C-1")
    assert A == C
    full = ks.full_softmax_fwd_bwd(dev(W, torch.bfloat16), dev(X, torch.bfloat16), dev(y), 30.0, 1.0, unit_rows=True)
    torch.cuda.synchronize()
    # same kernels (the last mode run above is the unit-rows one), same active list => bit-identical
    assert torch.equal(full["loss_per_sample"], out["loss_per_sample"])
    assert torch.equal(full["dX"], out["dX"])
    assert torch.equal(full["dW"], out["dW_active"])
    ofull = orc.full_softmax_fwd_bwd(W, X, y, 30.0, 1.0)
    assert abs(float(full["loss_mean"].item()) - ofull["loss"]) <= LOSS_RTOL * ofull["loss"]
    _check_full(full, ofull, W, X, y, 30.0, 1.0, "full K=C-1")


def _check_full(full, ref, W, X, y, scale, grad_scale, tag):
    """Full softmax: every row of dX and of the dense dW [C, D] against the oracle's full-softmax function."""
    lse = ref["loss_i"] + scale * (X.astype(np.float64) * W[y].astype(np.float64)).sum(axis=1)   # loss_i = lse - z_target
    f_dx, f_dw = grad_floors(W, X, np.asarray(y), lse, scale, grad_scale / X.shape[0])
    check_rows(full["dX"].cpu().numpy(), ref["dX"], f_dx, f"{tag} dX")
    check_rows(full["dW"].cpu().numpy(), ref["dW"], f_dw, f"{tag} dW")


@pytest.mark.parametrize("unit_rows", [False, True])
def test_full_softmax_on_20000_class_slice(ks, orc, unit_rows):
    C, D, B = 20_000, 512, 64
    W = synth.unit_rows(0, synth.TID_W, C, D, bf16=True)
    X = synth.unit_rows(0, synth.TID_X, B, D, bf16=True)
    y = synth.labels_uniform(0, B, C)
    full = ks.full_softmax_fwd_bwd(dev(W, torch.bfloat16), dev(X, torch.bfloat16), dev(y), 30.0, 1.0, unit_rows=unit_rows)
    torch.cuda.synchronize()
    assert int(full["dev_status"].item()) == 0
    ref = orc.full_softmax_fwd_bwd(W, X, y, 30.0, 1.0)
    assert abs(float(full["loss_mean"].item()) - ref["loss"]) <= LOSS_RTOL * ref["loss"]
    _check_full(full, ref, W, X, y, 30.0, 1.0, f"full 20k unit_rows={unit_rows}")


@pytest.mark.parametrize("unit_rows", [False, True])
def test_fwd_bwd_is_deterministic_and_softmax_invariants_hold(ks, orc, unit_rows):
    cfg = synth.CONFIGS["small"]
    W, X = synth.make_WX(cfg)
    y = synth.make_labels(cfg)
    G = synth.graph_synthetic(1, cfg["C"], cfg["K"])
    args = (dev(W, torch.bfloat16), dev(X, torch.bfloat16), dev(y), dev(G), cfg["M"], 30.0, 1.0)
    o1 = ks.knn_softmax_fwd_bwd(*args, unit_rows=unit_rows)
    o2 = ks.knn_softmax_fwd_bwd(*args, unit_rows=unit_rows)
    torch.cuda.synchronize()
    for k in ("active_idx", "n_active", "target_pos", "loss_per_sample", "loss_mean", "dX", "dW_active"):
        n = int(o1["n_active"].item()) if k == "dW_active" else None
        assert torch.equal(o1[k][:n], o2[k][:n]), k
    A = int(o1["n_active"].item())
    # sum_a dZ_ia = 0 => column sums of dW_active vanish (up to bf16 rounding of dZ)
    dW = o1["dW_active"][:A].double()
    assert dW.sum(dim=0).abs().max().item() <= 1e-3 * dW.abs().sum(dim=0).max().item()


def test_unit_rows_promise_with_longer_rows_still_gives_the_same_function(ks, orc):
    # rows 15 % longer than promised: logits reach 1.32 * scale, the fixed reference only shifts the exponents
    # (half of the samples sit near their class weight, so that some logits do exceed the scale)
    C, D, B, K, M = 6_000, 256, 300, 8, 1_500
    W = synth.bf16_round(1.15 * synth.unit_rows(11, synth.TID_W, C, D))
    y = synth.labels_uniform(11, B, C)
    X = synth.features_near_labels(11, W / 1.15, y, sigma=0.6)
    X[1::2] = synth.unit_rows(11, synth.TID_X, B, D)[1::2]
    X = synth.bf16_round(1.15 * X)
    assert (30.0 * (X * W[y]).sum(axis=1)).max() > 31.0
    G = synth.graph_synthetic(11, C, K, locality=3)
    run_and_compare(ks, orc, W, X, y, G, C, M, tag="long rows", modes=(True,))


def test_unit_rows_promise_broken_beyond_the_exponent_range_is_flagged(ks, orc):
    # rows of norm 2 at scale 40: target logits near 160, exp(160 - 40) overflows
    C, D, B, K, M = 2_000, 128, 64, 4, 512
    W0 = synth.unit_rows(12, synth.TID_W, C, D)
    y = synth.labels_uniform(12, B, C)
    X = synth.bf16_round(2.0 * synth.features_near_labels(12, W0, y, sigma=0.05))
    W = synth.bf16_round(2.0 * W0)
    out = ks.knn_softmax_fwd_bwd(dev(W, torch.bfloat16), dev(X, torch.bfloat16), dev(y), dev(synth.graph_synthetic(12, C, K)),
                                 M, 40.0, unit_rows=True)
    torch.cuda.synchronize()
    assert int(out["dev_status"].item()) & ks.KS_DEV_RANGE
    # without the promise the same inputs are handled
    out = ks.knn_softmax_fwd_bwd(dev(W, torch.bfloat16), dev(X, torch.bfloat16), dev(y), dev(synth.graph_synthetic(12, C, K)),
                                 M, 40.0)
    torch.cuda.synchronize()
    assert int(out["dev_status"].item()) == 0 and bool(torch.isfinite(out["loss_mean"]).all())


def test_bad_label_sets_flag_and_stays_in_bounds(ks, orc):
    C, D, B, K, M = 1000, 64, 8, 4, 64
    W = synth.unit_rows(0, synth.TID_W, C, D, bf16=True)
    X = synth.unit_rows(0, synth.TID_X, B, D, bf16=True)
    y = synth.labels_uniform(0, B, C)
    y[3] = C + 5
    out = ks.knn_softmax_fwd_bwd(dev(W, torch.bfloat16), dev(X, torch.bfloat16), dev(y), dev(synth.graph_synthetic(0, C, K)),
                                 M, 30.0)
    torch.cuda.synchronize()
    assert int(out["dev_status"].item()) & ks.KS_DEV_BAD_LABEL


# ------------------------------------------------------------------------------------------------
# weight update
# ------------------------------------------------------------------------------------------------
def _check_apply(ks, orc, W, idx, dW, alpha, sorted_unique, n=None):
    Wm = dev(W)
    Wb = dev(synth.bf16_round(W), torch.bfloat16)
    Wb0 = Wb.clone()
    n_dev = None if n is None else dev(np.array([n], dtype=np.int32))
    st = ks.apply_weight_grad(Wm, Wb, dev(idx), n_dev, dev(dW), alpha, idx_sorted_unique=sorted_unique)
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    nn = idx.shape[0] if n is None else n
    eWm, _ = orc.apply_weight_grad(W, idx[:nn], dW[:nn], alpha)
    got = Wm.cpu().numpy()
    touched = np.zeros(W.shape[0], dtype=bool)
    touched[idx[:nn]] = True
    assert (got[~touched] == W[~touched]).all()                       # untouched rows bit-unchanged
    assert torch.equal(Wb[torch.from_numpy(~touched).cuda()], Wb0[torch.from_numpy(~touched).cuda()])
    # fp32 update vs the oracle's fp64 sum: one rounding of the result plus the error of an fp32 sum of
    # `mult` terms, bounded by mult * 2^-24 * |alpha| * sum |terms|
    mult = np.bincount(idx[:nn], minlength=W.shape[0]).astype(np.float64)
    abssum = np.zeros(W.shape, dtype=np.float64)
    np.add.at(abssum, idx[:nn], np.abs(dW[:nn]).astype(np.float64))
    bound = 2.0 ** -23 * np.abs(eWm) + (mult[:, None] * 2.0 ** -24) * abs(alpha) * abssum + 1e-12
    assert (np.abs(got.astype(np.float64) - eWm) <= bound)[touched].all()
    # the bf16 copy is exactly the round-to-nearest-even of the master the GPU produced
    gb = Wb.view(torch.int16).cpu().numpy().view(np.uint16)
    assert (gb[touched] == synth.bf16_bits(got[touched])).all()


def test_apply_sorted_unique(ks, orc):
    C, D = 5000, 512
    W = synth.unit_rows(1, synth.TID_W, C, D)
    idx = np.sort(synth.class_permutation(1, C)[:1234]).astype(np.int32)
    dW = synth.grad_rows(1, idx.shape[0], D)
    _check_apply(ks, orc, W, idx, dW, -0.05, True)
    _check_apply(ks, orc, W, idx, dW, -0.05, True, n=1000)   # device-side count below n_max
    _check_apply(ks, orc, W, idx, dW, -0.05, False)          # the general path gives the same


@pytest.mark.parametrize("n,D,hi", [(300, 96, 40), (5000, 128, 700), (9000, 64, 3), (1, 32, 1)])
def test_apply_with_repeated_indices(ks, orc, n, D, hi):
    C = 1000
    rng = np.random.default_rng(n)
    W = synth.unit_rows(2, synth.TID_W, C, D)
    idx = rng.integers(0, hi, n).astype(np.int32)
    dW = synth.grad_rows(2, n, D)
    _check_apply(ks, orc, W, idx, dW, 0.25, False)
    # deterministic: a second run on the same inputs gives the same bits
    Wm1, Wm2 = dev(W), dev(W)
    ks.apply_weight_grad(Wm1, None, dev(idx), None, dev(dW), 0.25, False)
    ks.apply_weight_grad(Wm2, None, dev(idx), None, dev(dW), 0.25, False)
    torch.cuda.synchronize()
    assert torch.equal(Wm1, Wm2)


def test_apply_flags_broken_promise_and_bad_index(ks, orc):
    C, D = 100, 32
    W = synth.unit_rows(3, synth.TID_W, C, D)
    dW = synth.grad_rows(3, 4, D)
    st = ks.apply_weight_grad(dev(W), None, dev(np.array([1, 5, 5, 9], dtype=np.int32)), None, dev(dW), 1.0, True)
    torch.cuda.synchronize()
    assert int(st.item()) & ks.KS_DEV_IDX_NOT_SORTED
    st = ks.apply_weight_grad(dev(W), None, dev(np.array([1, 5, 100, 9], dtype=np.int32)), None, dev(dW), 1.0, False)
    torch.cuda.synchronize()
    assert int(st.item()) & ks.KS_DEV_BAD_INDEX


# ------------------------------------------------------------------------------------------------
# graph build
# ------------------------------------------------------------------------------------------------
def _check_graph(ks, orc, W, K, bf16, rows=None, tag=""):
    print(f"[graph] {tag} C={W.shape[0]} D={W.shape[1]} K={K} bf16={bf16}", flush=True)
    Wd = dev(W, torch.bfloat16) if bf16 else dev(W)
    g, s = ks.knn_graph_build(Wd, K, want_sims=True)
    torch.cuda.synchronize()
    g, s = g.cpu().numpy(), s.cpu().numpy()
    eg, es = orc.graph_bruteforce(W, K, rows)
    if rows is not None:
        g, s = g[rows], s[rows]
    assert (g == eg).all(), f"{(g != eg).any(axis=1).sum()} rows differ"
    assert (s == es.astype(np.float32)).all()
    return g


def test_graph_tiny_config_full_brute_force(ks, orc):
    cfg = synth.CONFIGS["tiny"]                       # C=10,000, D=128 fp32 input, K=8
    W = synth.unit_rows(0, synth.TID_W, cfg["C"], cfg["D"])
    _check_graph(ks, orc, W, cfg["K"], bf16=False, tag="tiny fp32")
    _check_graph(ks, orc, synth.bf16_round(W), cfg["K"], bf16=True, tag="tiny bf16")


@pytest.mark.parametrize("C,D,K,bf16", [(64, 32, 10, True), (1000, 32, 31, False), (5, 32, 4, True), (2, 32, 1, False),
                                        (300, 64, 100, True), (1500, 96, 64, True), (1500, 96, 128, False)])
def test_graph_exact_ties_one_hot_rows(ks, orc, C, D, K, bf16):
    W = np.zeros((C, D), dtype=np.float32)
    W[np.arange(C), np.arange(C) % D] = 1.0
    g = _check_graph(ks, orc, W, K, bf16, tag="one-hot")
    for i in (0, C - 1):
        same = [j for j in range(C) if j % D == i % D and j != i]
        other = [j for j in range(C) if j % D != i % D]
        assert g[i].tolist() == (same + other)[:K]


def test_graph_integer_entries_many_ties_and_twins(ks, orc):
    rng = np.random.default_rng(0)
    C, D, K = 2500, 32, 33
    W = rng.integers(-2, 3, (C, D)).astype(np.float32)
    W[1200] = W[7]
    W[1900] = W[7]
    g = _check_graph(ks, orc, W, K, True, tag="integers")
    assert g[7, 0] == 1200 and g[7, 1] == 1900 and g[1200, 0] == 7


def test_graph_clustered_rows_ragged_size(ks, orc):
    C, D, K = 20_011, 256, 32
    W = synth.clustered_rows(5, C, D, n_centres=257, bf16=True)
    rows = np.sort(synth.class_permutation(5, C)[:300]).astype(np.int32)
    _check_graph(ks, orc, W, K, True, rows=rows, tag="clustered")


@pytest.mark.parametrize("C,D,K,bf16,kind", [(3001, 128, 64, True, "unit"), (2500, 256, 100, True, "unit"),
                                             (5003, 512, 32, False, "unit"), (4000, 128, 32, True, "integers"),
                                             (3000, 256, 70, False, "integers"), (6000, 512, 16, True, "clustered")])
def test_graph_sweep_kernel_buffer_sizes_and_ties(ks, orc, C, D, K, bf16, kind):
    """The stationary-operand recall kernel (D = 128, 256, 512) with every candidate-buffer configuration (k' = 48, 64,
    128 with 256-entry buffers; k' = 256 with 512-entry buffers), on rows with few distinct similarities (small integer
    entries, twins: the cuts of the buffers meet many equal keys) and on clustered rows."""
    if kind == "unit":
        W = synth.unit_rows(9, synth.TID_W, C, D, bf16=bf16)
    elif kind == "integers":
        W = np.random.default_rng(C + D).integers(-1, 2, (C, D)).astype(np.float32)
        W[C // 2] = W[3]
        W[C - 1] = W[3]
    else:
        W = synth.clustered_rows(9, C, D, n_centres=97, bf16=bf16)
    rows = np.sort(synth.class_permutation(9, C)[:200]).astype(np.int32)
    rows[0] = 3
    rows = np.unique(rows)
    _check_graph(ks, orc, W, K, bf16, rows=rows, tag=f"sweep kernel {kind}")


@pytest.mark.parametrize("C,D,K,bf16,kind", [(6400, 128, 32, True, "unit"), (7000, 128, 8, True, "unit"),
                                             (8330, 256, 16, False, "unit"), (6913, 512, 32, True, "clustered"),
                                             (25_000, 128, 32, True, "unit"), (50_011, 128, 16, True, "clustered"),
                                             (6400, 128, 32, True, "integers"), (9000, 256, 64, True, "unit"),
                                             (12_345, 128, 40, False, "clustered"), (7000, 512, 64, True, "integers")])
def test_graph_every_similarity_computed_once(ks, orc, C, D, K, bf16, kind):
    """The recall pass that uses the symmetry of the similarities (D = 128, 256, 512, K <= 64): block, super-block and
    group counts that are odd, even and ragged (a last super-block of one, two and three blocks; groups of one, two and
    four super-blocks), all three values of k' (48, 64, 128), clustered rows, and rows with so many equal similarities
    that the fixed-size buffers overflow and the rows go to the exhaustive pass."""
    if kind == "unit":
        W = synth.unit_rows(11, synth.TID_W, C, D, bf16=bf16)
    elif kind == "integers":
        W = np.random.default_rng(C + D).integers(-1, 2, (C, D)).astype(np.float32)
        W[C // 2] = W[3]
        W[C - 1] = W[3]
    else:
        W = synth.clustered_rows(11, C, D, n_centres=97, bf16=bf16)
    n_rows = 400 if C <= 10_000 else 160
    rows = np.sort(synth.class_permutation(11, C)[:n_rows]).astype(np.int32)
    rows = np.unique(np.concatenate([rows, [0, 3, 255, 256, 767, 768, C // 2, C - 257, C - 2, C - 1]])).astype(np.int32)
    _check_graph(ks, orc, W, K, bf16, rows=rows, tag=f"symmetric recall {kind}")


def test_graph_tight_clusters_beside_lone_rows(ks, orc):
    """Rows that alternate, four by four, between tight clusters (hundreds of neighbours a few 1e-6 apart: no k' of a few
    dozen certifies the K-th one) and random directions (rows four apart share accumulator registers in the sweep and have
    nothing else in common).  The lists must be exact, and the build must not fall back on the exhaustive search for
    more than a handful of rows: uncertified rows are ranked again over everything the sweep kept for them."""
    C, D, K = 40_000, 128, 32
    rnd = synth.unit_rows(13, synth.TID_W, C, D).astype(np.float64)
    centres = synth.unit_rows(14, synth.TID_W, 64, D).astype(np.float64)
    idx = np.arange(C)
    W = np.where((((idx >> 2) & 1) == 0)[:, None], centres[idx % 64] + 0.1 * rnd, rnd)
    W = synth.bf16_round((W / np.sqrt((W * W).sum(axis=1, keepdims=True))).astype(np.float32))
    rows = np.unique(np.concatenate([np.sort(synth.class_permutation(13, C)[:150]), [0, 3, 4, 7, C - 1]])).astype(np.int32)
    Wd = dev(W, torch.bfloat16)
    ks.knn_graph_build(Wd, K)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    g, s = ks.knn_graph_build(Wd, K, want_sims=True)
    e1.record()
    torch.cuda.synchronize()
    print(f"[graph] tight clusters beside lone rows: {e0.elapsed_time(e1):.1f} ms", flush=True)
    assert e0.elapsed_time(e1) < 500.0   # (a few ms; with a thousand rows in the exhaustive search it would be seconds)
    eg, es = orc.graph_bruteforce(W, K, rows)
    assert (g.cpu().numpy()[rows] == eg).all() and (s.cpu().numpy()[rows] == es.astype(np.float32)).all()


@pytest.mark.parametrize("C", [6000, 9000])   # the plain recall pass; the one that computes every similarity once
def test_graph_is_deterministic(ks, orc, C):
    W = synth.unit_rows(6, synth.TID_W, C, 128, bf16=True)
    g1, s1 = ks.knn_graph_build(dev(W, torch.bfloat16), 16, want_sims=True)
    g2, s2 = ks.knn_graph_build(dev(W, torch.bfloat16), 16, want_sims=True)
    torch.cuda.synchronize()
    assert torch.equal(g1, g2) and torch.equal(s1, s2)
    assert (np.diff(s1.cpu().numpy(), axis=1) <= 0).all()


def test_gather_rows(ks, orc):
    C, D, M = 3000, 512, 700
    W = synth.unit_rows(7, synth.TID_W, C, D, bf16=True)
    idx = np.full(M, -1, dtype=np.int32)
    idx[:600] = np.sort(synth.class_permutation(7, C)[:600])
    out = ks.knn_gather_rows(dev(W, torch.bfloat16), dev(idx), dev(np.array([600], dtype=np.int32)))
    torch.cuda.synchronize()
    assert (out[:600].float().cpu().numpy() == W[idx[:600]]).all()


# ------------------------------------------------------------------------------------------------
# the whole step in one call (update inside the dW kernel)
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name,unit_rows,want_dW", [("small", True, False), ("small", False, True), ("tiny", False, False)])
def test_one_call_step_equals_forward_backward_then_update(ks, orc, name, unit_rows, want_dW):
    """Bit for bit: master weights, 16-bit copy, dX, loss -- the fused update does the same fused multiply-add on the
    same fp32 gradient value.  `tiny` has D = 128 in fp32 inputs rounded to bf16 (stationary-operand path too)."""
    cfg = synth.CONFIGS[name]
    C, D, B, K, M, scale = cfg["C"], cfg["D"], cfg["B"], cfg["K"], cfg["M"], cfg["scale"]
    W, X = synth.make_WX(cfg)
    W = synth.bf16_round(W)
    y = synth.make_labels(cfg)
    G = synth.graph_synthetic(cfg["seed"], C, K)
    gs, alpha = 128.0, -0.05 / 128.0
    Wb, Xb, yd, Gd = dev(W, torch.bfloat16), dev(synth.bf16_round(X), torch.bfloat16), dev(y), dev(G)
    # two calls
    Wm1, Wb1 = dev(W), Wb.clone()
    a = ks.knn_softmax_fwd_bwd(Wb1, Xb, yd, Gd, M, scale, gs, unit_rows=unit_rows)
    ks.apply_weight_grad(Wm1, Wb1, a["active_idx"], a["n_active"], a["dW_active"], alpha, idx_sorted_unique=True)
    # one call
    Wm2, Wb2 = dev(W), Wb.clone()
    b = ks.knn_softmax_fwd_bwd_update(Wm2, Wb2, Xb, yd, Gd, M, scale, gs, alpha, unit_rows=unit_rows, want_dW=want_dW)
    torch.cuda.synchronize()
    assert int(a["dev_status"].item()) == 0 and int(b["dev_status"].item()) == 0
    assert torch.equal(a["active_idx"], b["active_idx"]) and torch.equal(a["target_pos"], b["target_pos"])
    assert torch.equal(a["loss_per_sample"], b["loss_per_sample"]) and torch.equal(a["dX"], b["dX"])
    assert torch.equal(Wm1, Wm2) and torch.equal(Wb1, Wb2)
    A = int(a["n_active"].item())
    assert not torch.equal(Wm2, dev(W))                           # something was updated
    if want_dW:
        assert torch.equal(a["dW_active"][:A], b["dW_active"][:A])
    else:
        assert b["dW_active"] is None
    # and against the oracle: the change of the touched rows
    active, A_ref, tpos = orc.select_active(y, G, C, M)
    active = active[:A_ref]
    assert A == A_ref and (a["active_idx"][:A].cpu().numpy() == active).all()
    assert (a["target_pos"].cpu().numpy() == tpos).all()
    ref = orc.knn_softmax_fwd_bwd(W, synth.bf16_round(X), active, tpos, scale, gs)
    eW, _ = orc.apply_weight_grad(W, active, ref["dWA"].astype(np.float32), alpha, want_bf16=False)
    got = Wm2[torch.from_numpy(active.astype(np.int64)).cuda()].cpu().numpy().astype(np.float64)
    assert rel_fro(got - W[active], eW[active].astype(np.float64) - W[active]) <= GRAD_RTOL
    # row by row: the change of every touched row is alpha times the oracle's gradient row, up to the rounding of the
    # stored logit gradient and one fp32 rounding of the updated row
    _, f_dw = grad_floors(W[active], synth.bf16_round(X), tpos, ref["lse"], scale, gs / B)
    f_dw = f_dw + 2.0 ** -24 * np.linalg.norm(W[active].astype(np.float64), axis=1) / abs(alpha)
    check_rows((got - W[active]) / alpha, ref["dWA"], f_dw, f"{name} weight change / alpha")
    rest = np.setdiff1d(np.arange(C), active)
    assert (Wm2.cpu().numpy()[rest] == W[rest]).all()


@pytest.mark.parametrize("C,D,B,K,M", [(3000, 64, 70, 8, 300), (5000, 192, 200, 12, 1000), (2000, 320, 33, 4, 130)])
def test_one_call_step_ragged_shapes(ks, orc, C, D, B, K, M):
    """D below and between the tile widths, B and the active count not multiples of anything: the update inside the
    dW kernel against forward/backward followed by the stand-alone update, bit for bit."""
    W = synth.unit_rows(7, synth.TID_W, C, D, bf16=True)
    X = synth.unit_rows(7, synth.TID_X, B, D, bf16=True)
    y = synth.labels_uniform(7, B, C)
    G = synth.graph_synthetic(7, C, K)
    Wb, Xb, yd, Gd = dev(W, torch.bfloat16), dev(X, torch.bfloat16), dev(y), dev(G)
    for unit_rows in (False, True):
        Wm1, Wb1 = dev(W), Wb.clone()
        a = ks.knn_softmax_fwd_bwd(Wb1, Xb, yd, Gd, M, 25.0, 4.0, unit_rows=unit_rows)
        ks.apply_weight_grad(Wm1, Wb1, a["active_idx"], a["n_active"], a["dW_active"], -0.02, idx_sorted_unique=True)
        Wm2, Wb2 = dev(W), Wb.clone()
        b = ks.knn_softmax_fwd_bwd_update(Wm2, Wb2, Xb, yd, Gd, M, 25.0, 4.0, -0.02, unit_rows=unit_rows)
        torch.cuda.synchronize()
        assert int(a["dev_status"].item()) == 0 and int(b["dev_status"].item()) == 0
        assert torch.equal(Wm1, Wm2) and torch.equal(Wb1, Wb2) and torch.equal(a["dX"], b["dX"])
        assert torch.equal(a["loss_mean"], b["loss_mean"]) and not torch.equal(Wm2, dev(W))


def test_one_call_step_on_a_shape_without_the_fused_update(ks, orc):
    """D = 96: the gradient is stored and the stand-alone update runs inside the same call."""
    C, D, B, K, M, scale = 3000, 96, 64, 8, 512, 20.0
    W = synth.unit_rows(6, synth.TID_W, C, D, bf16=True)
    X = synth.unit_rows(6, synth.TID_X, B, D, bf16=True)
    y = synth.labels_uniform(6, B, C)
    G = synth.graph_synthetic(6, C, K)
    Wb, Xb, yd, Gd = dev(W, torch.bfloat16), dev(X, torch.bfloat16), dev(y), dev(G)
    Wm1, Wb1 = dev(W), Wb.clone()
    a = ks.knn_softmax_fwd_bwd(Wb1, Xb, yd, Gd, M, scale, 1.0)
    ks.apply_weight_grad(Wm1, Wb1, a["active_idx"], a["n_active"], a["dW_active"], -0.1, idx_sorted_unique=True)
    Wm2, Wb2 = dev(W), Wb.clone()
    b = ks.knn_softmax_fwd_bwd_update(Wm2, Wb2, Xb, yd, Gd, M, scale, 1.0, -0.1)
    torch.cuda.synchronize()
    assert b["dW_active"] is not None and torch.equal(Wm1, Wm2) and torch.equal(Wb1, Wb2) and torch.equal(a["dX"], b["dX"])


# ------------------------------------------------------------------------------------------------
# the step on a selection computed earlier (the selection of the next batch can run beside the current step)
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name,unit_rows", [("small", True), ("small", False), ("tiny", True)])
def test_step_on_an_earlier_selection_equals_the_one_call_step(ks, orc, name, unit_rows):
    """knn_select_active on a second stream, then knn_softmax_fwd_bwd_update_selected on the first: master weights,
    16-bit copy, dX and losses equal the one-call step bit for bit; without W_master it returns the gradient rows of
    knn_softmax_fwd_bwd."""
    cfg = synth.CONFIGS[name]
    C, D, B, K, M, scale = cfg["C"], cfg["D"], cfg["B"], cfg["K"], cfg["M"], cfg["scale"]
    W, X = synth.make_WX(cfg)
    W = synth.bf16_round(W)
    y = synth.make_labels(cfg)
    G = synth.graph_synthetic(cfg["seed"], C, K)
    gs, alpha = 64.0, -0.03 / 64.0
    Wb, Xb, yd, Gd = dev(W, torch.bfloat16), dev(synth.bf16_round(X), torch.bfloat16), dev(y), dev(G)
    Wm1, Wb1 = dev(W), Wb.clone()
    a = ks.knn_softmax_fwd_bwd_update(Wm1, Wb1, Xb, yd, Gd, M, scale, gs, alpha, unit_rows=unit_rows)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        act, n, tp, st = ks.knn_select_active(yd, Gd, C, M, stream=side)
    done = torch.cuda.Event()
    done.record(side)
    torch.cuda.current_stream().wait_event(done)
    Wm2, Wb2 = dev(W), Wb.clone()
    b = ks.knn_softmax_fwd_bwd_update_selected(Wm2, Wb2, Xb, act, n, tp, scale, gs, alpha, unit_rows=unit_rows)
    torch.cuda.synchronize()
    assert int(st.item()) == 0 and int(a["dev_status"].item()) == 0 and int(b["dev_status"].item()) == 0
    assert torch.equal(act, a["active_idx"]) and torch.equal(tp, a["target_pos"])
    assert torch.equal(a["loss_per_sample"], b["loss_per_sample"]) and torch.equal(a["loss_mean"], b["loss_mean"])
    assert torch.equal(a["dX"], b["dX"]) and torch.equal(Wm1, Wm2) and torch.equal(Wb1, Wb2)
    assert not torch.equal(Wm2, dev(W))
    # no update: the gradient rows of the plain forward/backward call
    c = ks.knn_softmax_fwd_bwd(Wb, Xb, yd, Gd, M, scale, gs, unit_rows=unit_rows)
    d = ks.knn_softmax_fwd_bwd_update_selected(None, Wb, Xb, act, n, tp, scale, gs, 0.0, unit_rows=unit_rows)
    torch.cuda.synchronize()
    A = int(n.item())
    assert torch.equal(c["dW_active"][:A], d["dW_active"][:A]) and torch.equal(c["dX"], d["dX"])


@pytest.mark.parametrize("name,shape,unit_rows,in_place,trusted", [
    ("small", None, True, True, False), ("small", None, False, False, False), ("tiny", None, True, False, False),
    ("small", None, True, False, True), ("tiny", None, False, False, True),
    ("the cut bites", dict(C=20_000, D=128, B=128, K=16, M=700, labels="zipf"), True, True, False),
    ("the cut bites", dict(C=20_000, D=128, B=128, K=16, M=700, labels="zipf"), True, False, True),
    ("D = 96", dict(C=5_000, D=96, B=70, K=9, M=300), False, False, False),
    ("D = 96", dict(C=5_000, D=96, B=70, K=9, M=300), False, False, True),
    ("the table path", dict(C=400_000, D=128, B=64, K=8, M=1_024), True, True, False),
    ("one sample", dict(C=300, D=64, B=1, K=3, M=4), False, True, False),
    ("lists as long as M allows", dict(C=3_000, D=128, B=5, K=7, M=8), True, False, True),
    ("batch not a power of two, 393,216 classes", dict(C=393_216, D=64, B=100, K=5, M=600), True, False, True),
    ("a large batch", dict(C=200_000, D=128, B=3000, K=32, M=65_536, labels="zipf"), True, False, True),
    ("a large batch, the cut bites", dict(C=200_000, D=128, B=4096, K=32, M=20_000), True, True, False)])
def test_selection_of_the_next_batch_rides_along_with_the_step(ks, orc, name, shape, unit_rows, in_place, trusted):
    """A loop of knn_softmax_fwd_bwd_update_selected_next calls (the step on this batch's list, the next batch's list
    made by extra workgroups of the same launches) against a loop of one-call steps on the same batches: every
    batch's active list, target positions, losses and dX, and the weights after the last step, bit for bit.  With the
    list buffers reused in place and with separate ones; D a multiple of 64 (the selection rides along) and not, and
    more classes than one workgroup's bitmap holds (then it follows the step); a batch whose lists exceed M; and with
    the list declared trusted (read in place, no validating copy: separate buffers are then required)."""
    cfg = dict(synth.CONFIGS["tiny"], **shape) if shape else synth.CONFIGS[name]
    C, D, B, K, M, scale = cfg["C"], cfg["D"], cfg["B"], cfg["K"], cfg["M"], cfg["scale"]
    W, X = synth.make_WX(cfg)
    W = synth.bf16_round(W)
    G = synth.graph_synthetic(cfg["seed"], C, K)
    gs, alpha = 64.0, -0.03 / 64.0
    Xb, Gd = dev(synth.bf16_round(X), torch.bfloat16), dev(G)
    n_steps = 4
    ys = [dev(synth.make_labels(cfg, seed=cfg["seed"] + 17 * t)) for t in range(n_steps + 1)]
    # reference: one-call steps
    Wm1, Wb1 = dev(W), dev(W, torch.bfloat16)
    ref = []
    for t in range(n_steps):
        a = ks.knn_softmax_fwd_bwd_update(Wm1, Wb1, Xb, ys[t], Gd, M, scale, gs, alpha, unit_rows=unit_rows)
        torch.cuda.synchronize()
        assert int(a["dev_status"].item()) == 0
        ref.append({k: a[k].clone() for k in ("active_idx", "n_active", "target_pos", "loss_per_sample", "loss_mean", "dX")})
    # the loop under test
    Wm2, Wb2 = dev(W), dev(W, torch.bfloat16)
    act, n, tp, st = ks.knn_select_active(ys[0], Gd, C, M)
    cur = dict(active_idx=act, n_active=n, target_pos=tp)
    spare = dict(active_idx=torch.empty_like(act), n_active=torch.empty_like(n), target_pos=torch.empty_like(tp))
    for t in range(n_steps):
        print(f"[case] {name}: step {t} with the selection of batch {t + 1} riding along", flush=True)
        torch.cuda.synchronize()
        assert torch.equal(cur["active_idx"], ref[t]["active_idx"]) and torch.equal(cur["n_active"], ref[t]["n_active"])
        assert torch.equal(cur["target_pos"], ref[t]["target_pos"])
        b, nxt = ks.knn_softmax_fwd_bwd_update_selected_next(Wm2, Wb2, Xb, cur["active_idx"], cur["n_active"], cur["target_pos"],
                                                             ys[t + 1], Gd, scale, gs, alpha,
                                                             next_out=None if in_place else spare, unit_rows=unit_rows,
                                                             trusted_list=trusted)
        torch.cuda.synchronize()
        assert int(b["dev_status"].item()) == 0
        assert torch.equal(b["loss_per_sample"], ref[t]["loss_per_sample"]) and torch.equal(b["loss_mean"], ref[t]["loss_mean"])
        assert torch.equal(b["dX"], ref[t]["dX"])
        if not in_place:
            cur, spare = nxt, cur
    assert torch.equal(Wm1, Wm2) and torch.equal(Wb1, Wb2) and int(st.item()) == 0
    # the list left by the last call is the one of the batch after it
    act_l, n_l, tp_l, _ = ks.knn_select_active(ys[n_steps], Gd, C, M)
    torch.cuda.synchronize()
    assert torch.equal(cur["active_idx"], act_l) and torch.equal(cur["n_active"], n_l) and torch.equal(cur["target_pos"], tp_l)


def test_headline_loop_replayed_from_a_hip_graph(ks):
    """The library allocates nothing, clears nothing with memset and never synchronises, so a training loop can capture
    its calls: two steps of the headline loop (list A -> list B -> list A) captured once and replayed three times, the
    labels of the coming batches copied into fixed buffers and other eager work done between the replays; weights, 16-bit
    copy and the last list against six eager one-call steps, bit for bit, after every replay."""
    cfg = synth.CONFIGS["small"]
    C, D, B, K, M, scale = cfg["C"], cfg["D"], cfg["B"], cfg["K"], cfg["M"], cfg["scale"]
    W, X = synth.make_WX(cfg)
    W = synth.bf16_round(W)
    G = synth.graph_synthetic(cfg["seed"], C, K)
    gs, alpha = 64.0, -0.03 / 64.0
    Xb, Gd = dev(synth.bf16_round(X), torch.bfloat16), dev(G)
    ys = [dev(synth.make_labels(cfg, seed=cfg["seed"] + 5 * t)) for t in range(7)]
    Wm1, Wb1 = dev(W), dev(W, torch.bfloat16)
    ref_W = []
    for t in range(6):
        a = ks.knn_softmax_fwd_bwd_update(Wm1, Wb1, Xb, ys[t], Gd, M, scale, gs, alpha, unit_rows=True)
        if t % 2 == 1:
            torch.cuda.synchronize()
            ref_W.append((Wm1.clone(), Wb1.clone()))
    assert int(a["dev_status"].item()) == 0
    Wm2, Wb2 = dev(W), dev(W, torch.bfloat16)
    act, n, tp, _ = ks.knn_select_active(ys[0], Gd, C, M)
    L0 = dict(active_idx=act, n_active=n, target_pos=tp)
    L1 = {k: torch.empty_like(v) for k, v in L0.items()}
    Ya, Yb = torch.empty_like(ys[0]), torch.empty_like(ys[0])
    out = dict(loss_per_sample=torch.empty(B, dtype=torch.float32, device="cuda"),
               loss_mean=torch.empty(1, dtype=torch.float32, device="cuda"),
               dX=torch.empty((B, D), dtype=torch.float32, device="cuda"), dW_active=None,
               dev_status=torch.zeros(1, dtype=torch.int32, device="cuda"))
    ws = torch.empty(ks.knn_softmax_selected_next_workspace(C, D, B, K, M), dtype=torch.uint8, device="cuda")

    def two_steps():
        ks.knn_softmax_fwd_bwd_update_selected_next(Wm2, Wb2, Xb, L0["active_idx"], L0["n_active"], L0["target_pos"], Ya, Gd, scale,
                                                    gs, alpha, next_out=L1, out=out, ws=ws, unit_rows=True, trusted_list=True)
        ks.knn_softmax_fwd_bwd_update_selected_next(Wm2, Wb2, Xb, L1["active_idx"], L1["n_active"], L1["target_pos"], Yb, Gd, scale,
                                                    gs, alpha, next_out=L0, out=out, ws=ws, unit_rows=True, trusted_list=True)

    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    Wm_keep, Wb_keep, L0_keep = Wm2.clone(), Wb2.clone(), {k: v.clone() for k, v in L0.items()}
    Ya.copy_(ys[1]); Yb.copy_(ys[2])
    print("[case] capturing two steps of the headline loop", flush=True)
    with torch.cuda.graph(graph):
        two_steps()
    # (capture runs nothing; the buffers are as before)
    Wm2.copy_(Wm_keep); Wb2.copy_(Wb_keep)
    for k in L0:
        L0[k].copy_(L0_keep[k])
    for r in range(3):
        Ya.copy_(ys[2 * r + 1]); Yb.copy_(ys[2 * r + 2])
        scratch = torch.randn(1 << 20, device="cuda").sum()      # eager work between the replays
        print(f"[case] replay {r}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        assert int(out["dev_status"].item()) == 0 and bool(torch.isfinite(scratch))
        assert torch.equal(Wm2, ref_W[r][0]) and torch.equal(Wb2, ref_W[r][1]), f"replay {r}"
    act6, n6, tp6, _ = ks.knn_select_active(ys[6], Gd, C, M)
    torch.cuda.synchronize()
    assert torch.equal(L0["active_idx"], act6) and torch.equal(L0["n_active"], n6) and torch.equal(L0["target_pos"], tp6)


def test_trusted_list_needs_buffers_of_its_own_for_the_next_list(ks):
    C, D, B, K, M = 2000, 128, 16, 4, 64
    W = torch.randn(C, D, device="cuda")
    Wb, X = W.to(torch.bfloat16), torch.randn(B, D, device="cuda").to(torch.bfloat16)
    y = torch.arange(B, dtype=torch.int32, device="cuda")
    G = torch.from_numpy(synth.graph_synthetic(0, C, K)).cuda()
    act, n, tp, _ = ks.knn_select_active(y, G, C, M)
    with pytest.raises(ks.KsError):
        ks.knn_softmax_fwd_bwd_update_selected_next(W, Wb, X, act, n, tp, y, G, 10.0, 1.0, -0.01, trusted_list=True)
    a, _ = ks.knn_softmax_fwd_bwd_update_selected_next(W.clone(), Wb.clone(), X, act, n, tp, y, G, 10.0, 1.0, -0.01)
    b = ks.knn_softmax_fwd_bwd_update_selected(W.clone(), Wb.clone(), X, act, n, tp, 10.0, 1.0, -0.01, trusted_list=True)
    torch.cuda.synchronize()
    assert torch.equal(a["dX"], b["dX"]) and torch.equal(a["loss_per_sample"], b["loss_per_sample"])


def test_step_on_a_broken_selection_is_flagged_and_stays_in_bounds(ks):
    C, D, B, M = 1000, 128, 16, 64
    W = torch.randn(C, D, device="cuda")
    Wb = W.to(torch.bfloat16)
    X = torch.randn(B, D, device="cuda").to(torch.bfloat16)
    act = torch.arange(M, dtype=torch.int32, device="cuda")
    act[3] = C + 5                                                # not a class
    tp = torch.zeros(B, dtype=torch.int32, device="cuda")
    tp[2] = 40                                                    # beyond the 32 valid entries
    n = torch.tensor([32], dtype=torch.int32, device="cuda")
    out = ks.knn_softmax_fwd_bwd_update_selected(W.clone(), Wb, X, act, n, tp, 10.0, 1.0, -0.01)
    torch.cuda.synchronize()
    stt = int(out["dev_status"].item())
    assert stt & ks.KS_DEV_BAD_INDEX and stt & ks.KS_DEV_BAD_LABEL
