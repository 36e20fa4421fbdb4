"""GPU parity of the normalisation inside the layer (Section 3.2.3, GPU pipeline step 2): row normalisation, the projection that brings
a gradient with respect to a normalised row back to the row itself, and the weight update through the
normalisation, each against the CPU oracle; then one whole step of the layer that keeps un-normalised fp32
weights (normalise X, forward/backward on the normalised copies, project dX, update W through the projection)
against the same composition of oracle calls, on small shapes and at the full size of the headline shard."""
import numpy as np
import pytest
import torch

import synth
from gradcheck import check_step_grads

pytestmark = pytest.mark.gpu

ULP32 = 2.0 ** -23


@pytest.fixture(scope="module")
def ks():
    import paper_2102_06025_amd as ks
    ks.lib()
    assert torch.cuda.is_available(), "these tests need the GPU"
    return ks


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t if dtype is None else t.to(dtype)


def bits(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def raw_rows(seed, n, D, bf16=False):
    """Rows with norms spread over about two decades (a layer's un-normalised weights or features)."""
    V = synth.unit_rows(seed, synth.TID_W, n, D).astype(np.float64)
    length = np.exp(2.3 * (synth.uniform01(seed, synth.TID_X, 0, n) * 2.0 - 1.0))
    V = (V * length[:, None]).astype(np.float32)
    return synth.bf16_round(V) if bf16 else V


def bf16_ulps_apart(a, b):
    """|a - b| in units of the last place for bf16 bit patterns of equal sign (adjacent patterns differ by 1)."""
    return np.abs(a.astype(np.int32) - b.astype(np.int32))


@pytest.mark.parametrize("n,D,bf16", [(1031, 512, True), (1031, 512, False), (257, 36, False), (64, 1280, True),
                                      (1, 4, False)])
def test_normalize_rows(ks, orc, n, D, bf16):
    print(f"[norm] normalize n={n} D={D} bf16={bf16}", flush=True)
    V = raw_rows(11, n, D, bf16)
    if n > 8:
        V[5] = 0.0                                   # a zero row stays zero, with inv_norm 0
    Vd = dev(V, torch.bfloat16) if bf16 else dev(V)
    Vh, inv = ks.knn_normalize_rows(Vd)
    torch.cuda.synchronize()
    _, eb, einv = orc.normalize_rows(V)
    got_inv = inv.cpu().numpy()
    assert np.abs(got_inv - einv).max() <= ULP32 * np.abs(einv).max()
    assert np.mean(got_inv == einv) > 0.99           # the fp64 sums differ only in their order
    gb = bits(Vh)
    assert np.mean(gb == eb) > 0.9999
    assert bf16_ulps_apart(gb, eb).max() <= 1
    if n > 8:
        assert got_inv[5] == 0.0 and (gb[5] & 0x7FFF == 0).all()
    # each output alone
    Vh2, none = ks.knn_normalize_rows(Vd, want_inv_norm=False)
    none2, inv2 = ks.knn_normalize_rows(Vd, want_bf16=False)
    torch.cuda.synchronize()
    assert none is None and none2 is None
    assert torch.equal(Vh2, Vh) and torch.equal(inv2, inv)


@pytest.mark.parametrize("n,D,bf16", [(1024, 512, True), (333, 260, False), (7, 2048, False)])
def test_norm_backward_rows(ks, orc, n, D, bf16):
    print(f"[norm] backward n={n} D={D} bf16={bf16}", flush=True)
    V = raw_rows(12, n, D, bf16)
    if n > 3:
        V[3] = 0.0
    G = synth.grad_rows(12, n, D)
    Vd = dev(V, torch.bfloat16) if bf16 else dev(V)
    out = ks.knn_norm_backward_rows(Vd, dev(G))
    torch.cuda.synchronize()
    ref = orc.norm_backward(V, G.astype(np.float64))
    got = out.cpu().numpy().astype(np.float64)
    # fp64 arithmetic on both sides; the result is rounded to fp32 once
    row_max = np.abs(ref).max(axis=1, keepdims=True)
    assert (np.abs(got - ref) <= ULP32 * np.maximum(row_max, 1e-30)).all()
    if n > 3:
        assert (got[3] == 0.0).all()
    # the projection is orthogonal to the row
    nz = np.abs(V).sum(axis=1) > 0
    dots = np.einsum("nd,nd->n", got[nz], V[nz].astype(np.float64))
    assert np.abs(dots).max() <= 1e-5 * np.abs(got).max() * np.abs(V).max() * D
    # in place
    Gd = dev(G)
    ks.knn_norm_backward_rows(Vd, Gd, out=Gd)
    torch.cuda.synchronize()
    assert torch.equal(Gd, out)


def _check_apply_normalized(ks, orc, W, idx, dW, alpha, sorted_unique, n=None, frac_equal=0.999):
    C, D = W.shape
    Wm = dev(W)
    Wh, inv = ks.knn_normalize_rows(Wm)
    Wh0, inv0 = Wh.clone(), inv.clone()
    n_dev = None if n is None else dev(np.array([n], dtype=np.int32))
    st = ks.apply_weight_grad_normalized(Wm, Wh, inv, dev(idx), n_dev, dev(dW), alpha, sorted_unique)
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    m = idx.shape[0] if n is None else n
    eW, eWb, einv = orc.apply_weight_grad_normalized(W, idx[:m], dW[:m], alpha)
    touched = np.unique(idx[:m])
    got = Wm.cpu().numpy()
    # both sides work in fp64 and round the new row to fp32 once: they differ where the two orders of the row
    # sums move a result across a rounding boundary
    assert np.abs(got[touched] - eW[touched]).max() <= 2 * ULP32 * np.abs(eW[touched]).max()
    if frac_equal is None:      # the sum over a class's rows was rounded to fp32 once before use
        frac_equal = 0.5
    assert np.mean(got[touched] == eW[touched]) > frac_equal
    got_inv = inv.cpu().numpy()
    assert np.abs(got_inv[touched] - einv[touched]).max() <= 2 * ULP32 * np.abs(einv[touched]).max()
    gb = bits(Wh)
    assert np.mean(gb[touched] == eWb[touched]) > frac_equal
    assert bf16_ulps_apart(gb[touched], eWb[touched]).max() <= 1
    # the normalised copy is the rounding of the GPU's own master row times its own inv_norm
    own = (got[touched].astype(np.float64) * got_inv[touched].astype(np.float64)[:, None]).astype(np.float32)
    assert np.mean(gb[touched] == synth.bf16_bits(own)) > frac_equal
    # rows that were not named keep their bits, in all three arrays
    rest = np.setdiff1d(np.arange(C), touched)
    assert (got[rest] == W[rest]).all()
    assert (gb[rest] == bits(Wh0)[rest]).all()
    assert (got_inv[rest] == inv0.cpu().numpy()[rest]).all()
    return got


def test_apply_normalized_sorted_unique(ks, orc):
    C, D = 5000, 512
    print(f"[norm] apply sorted C={C} D={D}", flush=True)
    W = raw_rows(1, C, D)
    idx = np.sort(synth.class_permutation(1, C)[:1234]).astype(np.int32)
    dW = synth.grad_rows(1, idx.shape[0], D)
    a = _check_apply_normalized(ks, orc, W, idx, dW, -0.5, True)
    _check_apply_normalized(ks, orc, W, idx, dW, -0.5, True, n=1000)     # device-side count below n_max
    b = _check_apply_normalized(ks, orc, W, idx, dW, -0.5, False)        # the general path gives the same rows
    assert (a == b).all()


@pytest.mark.parametrize("n,D,hi", [(300, 96, 40), (5000, 128, 700), (9000, 64, 3), (1, 32, 1), (700, 1040, 90)])
def test_apply_normalized_with_repeated_indices(ks, orc, n, D, hi):
    C = 1000
    print(f"[norm] apply repeated n={n} D={D} hi={hi}", flush=True)
    rng = np.random.default_rng(n)
    W = raw_rows(2, C, D)
    idx = rng.integers(0, hi, n).astype(np.int32)
    dW = synth.grad_rows(2, n, D)
    # the fp64 sum over a class's rows is rounded to fp32 once before it is used (a relative 2^-24 of the
    # gradient, times alpha, against the oracle's unrounded sum): last-place differences are expected here
    _check_apply_normalized(ks, orc, W, idx, dW, 0.25, False, frac_equal=None)
    Wm1, Wm2 = dev(W), dev(W)
    ks.apply_weight_grad_normalized(Wm1, None, None, dev(idx), None, dev(dW), 0.25, False)
    ks.apply_weight_grad_normalized(Wm2, None, None, dev(idx), None, dev(dW), 0.25, False)
    torch.cuda.synchronize()
    assert torch.equal(Wm1, Wm2)


def test_apply_normalized_flags_and_zero_rows(ks, orc):
    C, D = 100, 32
    W = raw_rows(3, C, D)
    W[7] = 0.0                                       # a zero master row: no direction to project on, left as it is
    dW = synth.grad_rows(3, 4, D)
    Wm = dev(W)
    st = ks.apply_weight_grad_normalized(Wm, None, None, dev(np.array([1, 5, 5, 9], dtype=np.int32)), None, dev(dW), 1.0,
                                         True)
    torch.cuda.synchronize()
    assert int(st.item()) & ks.KS_DEV_IDX_NOT_SORTED
    st = ks.apply_weight_grad_normalized(dev(W), None, None, dev(np.array([1, 5, 100, 9], dtype=np.int32)), None, dev(dW),
                                         1.0, False)
    torch.cuda.synchronize()
    assert int(st.item()) & ks.KS_DEV_BAD_INDEX
    for sorted_unique in (True, False):
        Wm = dev(W)
        Wh, inv = ks.knn_normalize_rows(Wm)
        st = ks.apply_weight_grad_normalized(Wm, Wh, inv, dev(np.array([2, 7, 9, 50], dtype=np.int32)), None, dev(dW), 1.0,
                                             sorted_unique)
        torch.cuda.synchronize()
        assert int(st.item()) == 0
        eW, eWb, einv = orc.apply_weight_grad_normalized(W, np.array([2, 7, 9, 50], dtype=np.int32), dW, 1.0)
        assert (Wm[7].cpu().numpy() == 0).all() and float(inv[7].item()) == 0.0 and (bits(Wh)[7] & 0x7FFF == 0).all()
        assert (eW[7] == 0).all() and einv[7] == 0.0
        assert np.abs(Wm.cpu().numpy() - eW).max() <= ULP32 * np.abs(eW).max()


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return np.linalg.norm(a - b) / np.linalg.norm(b)


def _layer_step(ks, orc, W, X, y, G, M, scale, grad_scale, lr):
    """One step of the layer with un-normalised fp32 weights and features, GPU against the oracle composition.
    Returns the relative errors (dX, weight change)."""
    C, D = W.shape
    alpha = -lr / grad_scale
    # ---- GPU
    Wm = dev(W)
    Wh, inv = ks.knn_normalize_rows(Wm)
    Xd = dev(X)
    Xh, _ = ks.knn_normalize_rows(Xd, want_inv_norm=False)
    out = ks.knn_softmax_fwd_bwd(Wh, Xh, dev(y), dev(G), M, scale, grad_scale, unit_rows=True)
    dX = ks.knn_norm_backward_rows(Xd, out["dX"])
    st = ks.apply_weight_grad_normalized(Wm, Wh, inv, out["active_idx"], out["n_active"], out["dW_active"], alpha,
                                         idx_sorted_unique=True)
    torch.cuda.synchronize()
    assert int(out["dev_status"].item()) == 0 and int(st.item()) == 0
    A = int(out["n_active"].item())
    # ---- oracle: the same composition in fp64 on the fp32 normalised rows (the GPU's contractions read their
    # bf16 roundings, which the gradient tolerance covers)
    W_hat, _, _ = orc.normalize_rows(W, want_bf16=False)
    X_hat, _, _ = orc.normalize_rows(X, want_bf16=False)
    active, A_ref, tpos = orc.select_active(y, G, C, M)
    assert A == A_ref and (out["active_idx"].cpu().numpy() == active).all()
    ref = orc.knn_softmax_fwd_bwd(W_hat, X_hat, active[:A], tpos, scale, grad_scale)
    loss = float(out["loss_mean"].item())
    assert abs(loss - ref["loss"]) <= 1e-3 * abs(ref["loss"])
    # the gradients with respect to the normalised rows, row by row, against the oracle working from the 16-bit
    # normalised rows the contractions read (the oracle's own rounding of its own normalised rows)
    _, Wb_o, _ = orc.normalize_rows(W[active[:A]])
    _, Xb_o, _ = orc.normalize_rows(X)
    W16 = np.zeros((C, D), dtype=np.float32)
    W16[active[:A]] = synth.bf16_to_f32(Wb_o)
    X16 = synth.bf16_to_f32(Xb_o)
    ref16 = orc.knn_softmax_fwd_bwd(W16, X16, active[:A], tpos, scale, grad_scale)
    check_step_grads(out["dX"].cpu().numpy(), out["dW_active"][:A].cpu().numpy(), ref16, W16[active[:A]], X16, tpos, scale,
                     grad_scale, tag="normalised layer")
    dX_ref = orc.norm_backward(X, ref["dX"])
    eW, _, einv = orc.apply_weight_grad_normalized(W, active[:A], ref["dWA"].astype(np.float32), alpha)
    e_dx = rel_fro(dX.cpu().numpy(), dX_ref)
    got = Wm.cpu().numpy()
    e_w = rel_fro(got[active[:A]].astype(np.float64) - W[active[:A]], eW[active[:A]].astype(np.float64) - W[active[:A]])
    rows = active[:A]
    # the refreshed normalised copy and inv_norm describe the GPU's own new master rows
    _, own_b, own_inv = orc.normalize_rows(got[rows])
    gb = bits(Wh[torch.from_numpy(rows.astype(np.int64)).cuda()])
    assert np.mean(gb == own_b) > 0.999 and bf16_ulps_apart(gb, own_b).max() <= 1
    assert np.abs(inv.cpu().numpy()[rows] - own_inv).max() <= 2 * ULP32 * own_inv.max()
    rest = np.setdiff1d(np.arange(C), rows)[:4096]
    assert (got[rest] == W[rest]).all()
    return e_dx, e_w, loss, ref["loss"], A


def test_layer_step_with_normalisation_small(ks, orc):
    cfg = synth.CONFIGS["small"]
    C, D, B, K, M, scale = cfg["C"], cfg["D"], cfg["B"], cfg["K"], cfg["M"], cfg["scale"]
    print(f"[norm] layer step small C={C} D={D} B={B}", flush=True)
    W = raw_rows(21, C, D)
    y = synth.make_labels(cfg)
    Xu = synth.features_near_labels(21, synth.unit_rows(21, synth.TID_W, C, D), y)
    Xu[B // 2:] = synth.unit_rows(22, synth.TID_X, B - B // 2, D)     # half the batch far from its label: losses of O(10)
    X = (Xu.astype(np.float64) * np.exp(synth.normal(21, synth.TID_X, 0, B))[:, None]).astype(np.float32)
    G = synth.graph_synthetic(21, C, K)
    e_dx, e_w, loss, loss_ref, A = _layer_step(ks, orc, W, X, y, G, M, scale, 128.0, 0.5)
    print(f"        A={A} loss={loss:.6f} ref={loss_ref:.6f} relF(dX)={e_dx:.2e} relF(W change)={e_w:.2e}", flush=True)
    assert e_dx <= 2e-2 and e_w <= 2e-2


def test_layer_step_with_normalisation_full_size(ks, orc):
    """The headline shard with un-normalised fp32 master weights; neighbour lists are an arithmetic pattern (the
    step does not depend on their being true neighbours, and the exact graph at this size has its own test)."""
    cfg = synth.CONFIGS["shard390k"]
    C, D, B, K, M, scale = cfg["C"], cfg["D"], cfg["B"], cfg["K"], cfg["M"], cfg["scale"]
    print(f"[norm] layer step shard390k C={C} D={D} B={B} K={K} M={M}", flush=True)
    W = raw_rows(22, C, D)
    y = synth.make_labels(cfg)
    X = raw_rows(23, B, D)
    c = np.arange(C, dtype=np.int64)[:, None]
    k = np.arange(K, dtype=np.int64)[None, :]
    G = ((c + 1 + (c * 2654435761 + k * 40503) % (C - 1)) % C).astype(np.int32)
    e_dx, e_w, loss, loss_ref, A = _layer_step(ks, orc, W, X, y, G, M, scale, 128.0, 0.5)
    print(f"        A={A} loss={loss:.6f} ref={loss_ref:.6f} relF(dX)={e_dx:.2e} relF(W change)={e_w:.2e}", flush=True)
    assert e_dx <= 2e-2 and e_w <= 2e-2
