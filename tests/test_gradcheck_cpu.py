"""The row-by-row gradient comparison (tests/gradcheck.py) must see what one norm over the whole matrix does not:
a stand-in for the GPU's result (the oracle's contraction redone in numpy with the logit gradient rounded to bf16,
which is what the HIP path stores) passes, and the same matrices with a row zeroed, two rows exchanged, stale rows
or a scaled row fail, although their whole-matrix error stays inside the tolerance."""
import numpy as np
import pytest

import synth
from gradcheck import GRAD_RTOL, check_rows, grad_floors, row_errors


@pytest.fixture(scope="module")
def case(orc):
    C, D, B, K, M, scale, gs = 20_000, 128, 256, 16, 4_096, 30.0, 128.0
    W = synth.unit_rows(3, synth.TID_W, C, D, bf16=True)
    X = synth.unit_rows(3, synth.TID_X, B, D, bf16=True)
    y = synth.labels_zipf(3, B, C)
    G = synth.graph_synthetic(3, C, K, locality=8)
    active, A, tpos = orc.select_active(y, G, C, M)
    ref = orc.knn_softmax_fwd_bwd(W, X, active[:A], tpos, scale, gs, want_P=True)
    W_A = W[active[:A]].astype(np.float64)
    g = gs / B
    dZ = ref["P"].copy()
    dZ[np.arange(B), tpos] -= 1.0
    dZ *= g
    dZ_stored = synth.bf16_round(dZ.astype(np.float32)).astype(np.float64)      # what the HIP path keeps
    dX = scale * dZ_stored @ W_A
    dW = scale * dZ_stored.T @ X.astype(np.float64)
    f_dx, f_dw = grad_floors(W_A, X, tpos, ref["lse"], scale, g)
    return dict(ref=ref, dX=dX, dW=dW, f_dx=f_dx, f_dw=f_dw, tpos=tpos, A=A, B=B)


def test_the_stand_in_passes_with_room(case):
    rx = check_rows(case["dX"], case["ref"]["dX"], case["f_dx"], "dX")
    rw = check_rows(case["dW"], case["ref"]["dWA"], case["f_dw"], "dW_A")
    assert rx["worst_ratio"] < 0.5 and rw["worst_ratio"] < 0.5


def test_floors_are_small_against_the_rows(case):
    # a floor of the order of the row would make the check blind; it stays a few per cent of the row's length
    ref = case["ref"]
    assert np.median(case["f_dw"] / np.linalg.norm(ref["dWA"], axis=1)) < 0.05
    assert np.median(case["f_dx"] / np.linalg.norm(ref["dX"], axis=1)) < 0.05


def _non_label_rows(case):
    rows = np.setdiff1d(np.arange(case["A"]), case["tpos"])
    assert len(rows) > case["A"] // 2
    return rows


def test_a_zeroed_row_fails_though_the_whole_matrix_norm_does_not_move(case):
    ref = case["ref"]["dWA"]
    rows = _non_label_rows(case)
    bad = case["dW"].copy()
    bad[rows[7]] = 0.0
    r = row_errors(bad, ref, case["f_dw"])
    assert r["rel_fro"] <= GRAD_RTOL                      # the old check would have passed
    assert r["n_bad"] == 1 and r["worst_row"] == rows[7]
    with pytest.raises(AssertionError):
        check_rows(bad, ref, case["f_dw"], "dW_A", quiet=True)


def test_many_wrong_rows_can_hide_in_the_whole_matrix_norm_but_not_here(case):
    ref = case["ref"]["dWA"]
    rows = _non_label_rows(case)
    bad = case["dW"].copy()
    # zero as many (short) non-label rows as the whole-matrix tolerance lets through: hundreds here, three
    # quarters of all rows at the headline shape
    norms = np.linalg.norm(ref[rows], axis=1)
    order = np.argsort(norms)
    n = int(np.searchsorted(np.cumsum(norms[order] ** 2), (0.015 * np.linalg.norm(ref)) ** 2))
    assert n >= 100
    bad[rows[order[:n]]] = 0.0
    r = row_errors(bad, ref, case["f_dw"])
    assert r["rel_fro"] <= GRAD_RTOL
    assert r["n_bad"] == n


def test_exchanged_rows_and_a_scaled_row_fail(case):
    ref = case["ref"]["dWA"]
    rows = _non_label_rows(case)
    bad = case["dW"].copy()
    bad[[rows[1], rows[2]]] = bad[[rows[2], rows[1]]]
    assert row_errors(bad, ref, case["f_dw"])["n_bad"] == 2
    bad = case["dW"].copy()
    bad[rows[3]] *= 1.1
    assert row_errors(bad, ref, case["f_dw"])["n_bad"] == 1
    # dX: a sample's row zeroed, two samples exchanged
    refx = case["ref"]["dX"]
    bad = case["dX"].copy()
    bad[5] = 0.0
    assert row_errors(bad, refx, case["f_dx"])["n_bad"] == 1
    bad = case["dX"].copy()
    bad[[8, 9]] = bad[[9, 8]]
    assert row_errors(bad, refx, case["f_dx"])["n_bad"] == 2


def test_shifted_rows_fail(case):
    # every row holds its neighbour's values (a gather-list slip)
    ref = case["ref"]["dWA"]
    bad = np.roll(case["dW"], 1, axis=0)
    assert row_errors(bad, ref, case["f_dw"])["n_bad"] > 0.95 * case["A"]
