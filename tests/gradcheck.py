"""Row-by-row comparison of the gradient matrices of the softmax layer (Section 3.2: "fc backward") with the
oracle's.  One norm over a whole matrix is nearly blind here: the rows of dW_A that belong to the batch's labels
carry almost all of its norm, so most other rows could be wrong without moving it.  Every row is therefore held to

    || got_r - ref_r ||_2  <=  rtol * || ref_r ||_2  +  floor_r

with rtol = 2e-2 (the stated tolerance) and floor_r the largest error that storing the logit gradient in bf16 can
cause in that row:

  * the GPU path stores dZ (or, in the one-sweep mode, exp(z - s) and X / sum) rounded to bf16: every term of a
    row's sum carries a relative error of at most EPS = 2^-8 (two roundings of half a unit in the last place, 2^-9 each);
  * row a of dW_A = s * sum_i dZ[i, a] * X[i, :]  =>  || error || <= EPS * s * sigma_max(X) * || dZ[:, a] ||_2;
  * row i of dX   = s * sum_a dZ[i, a] * W_A[a, :] =>  || error || <= EPS * s * sigma_max(W_A) * || dZ[i, :] ||_2,

sigma_max being the largest singular value.  One more term covers the logits being fp32 sums: the matrix cores add
the D products of a logit into an fp32 accumulator in D/16 steps of 16 products, each step rounding once at the size
of the partial sum (at most |x||w|), and the log-sum-exp and the exponent's argument are rounded as well, so a logit
is known to  dz = s * (D/16 + 4) * 2^-24 * |x| * |w|.  That moves a probability by the RELATIVE amount dz, far
below the bf16 term, except where it matters absolutely: the target entry g * (P_t - 1) of a confident sample
(P_t next to 1) moves by up to g * dz, and for such a sample the whole row of dX is of that size.  It adds
s * g * dz_i * |w_target|  to the floor of the sample's row of dX and  s * g * sum over the samples i of class a of
dz_i * |x_i|  to the floor of row a of dW_A.  The rest of the fp32 accumulation of the contractions is left to
rtol.  The floors are bounds on a tolerance, not expected values: they are evaluated here in numpy (fp64) from the
inputs and the oracle's log-sum-exp.  A zeroed, permuted or stale row
misses its reference by about its whole length and fails."""
import numpy as np

EPS_BF16_TWICE = 2.0 ** -8
EPS32 = 2.0 ** -24
GRAD_RTOL = 2e-2


def sigma_max(mat) -> float:
    """Largest singular value, from the Gram matrix of the shorter side (fp64)."""
    mat = np.asarray(mat, dtype=np.float64)
    gram = mat.T @ mat if mat.shape[0] >= mat.shape[1] else mat @ mat.T
    return float(np.sqrt(max(np.linalg.eigvalsh(gram)[-1], 0.0)))


def grad_floors(W_A, X, tpos, lse, scale, g, chunk=8192):
    """(floor_dX [B], floor_dW [A]) as defined in the module text.  W_A [A, D] the gathered rows, X [B, D], tpos [B]
    (negative: the sample has no target column here), lse [B] the log of the softmax denominator, g = grad_scale / B."""
    W_A = np.asarray(W_A, dtype=np.float64)
    X = np.asarray(X, dtype=np.float64)
    lse = np.asarray(lse, dtype=np.float64)
    A, B = W_A.shape[0], X.shape[0]
    row_sq = np.zeros(B)
    col = np.empty(A)
    for a0 in range(0, A, chunk):
        a1 = min(A, a0 + chunk)
        dZ = np.exp(scale * (X @ W_A[a0:a1].T) - lse[:, None])
        own = np.nonzero((tpos >= a0) & (tpos < a1))[0]
        dZ[own, tpos[own] - a0] -= 1.0
        dZ *= g
        row_sq += (dZ * dZ).sum(axis=1)
        col[a0:a1] = np.sqrt((dZ * dZ).sum(axis=0))
    floor_dX = EPS_BF16_TWICE * scale * sigma_max(W_A) * np.sqrt(row_sq)
    floor_dW = EPS_BF16_TWICE * scale * sigma_max(X) * col
    # fp32 evaluation of the target logit
    tpos = np.asarray(tpos)
    own = np.nonzero((tpos >= 0) & (tpos < A))[0]
    x_len = np.linalg.norm(X, axis=1)[own]
    w_len = np.linalg.norm(W_A[tpos[own]], axis=1)
    dz = scale * (X.shape[1] / 16.0 + 4.0) * EPS32 * x_len * w_len
    floor_dX[own] += scale * g * dz * w_len
    np.add.at(floor_dW, tpos[own], scale * g * dz * x_len)
    return floor_dX, floor_dW


def row_errors(got, ref, floor, rtol=GRAD_RTOL):
    """Per-row error, per-row allowance, and summary figures (dict)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    err = np.linalg.norm(got - ref, axis=1)
    tol = rtol * np.linalg.norm(ref, axis=1) + np.asarray(floor, dtype=np.float64)
    ratio = err / np.maximum(tol, 1e-300)
    worst = int(np.argmax(ratio)) if len(ratio) else 0
    den = np.linalg.norm(ref)
    return dict(err=err, tol=tol, n_bad=int((err > tol).sum()), worst_row=worst,
                worst_ratio=float(ratio[worst]) if len(ratio) else 0.0,
                max_abs=float(np.abs(got - ref).max()) if got.size else 0.0,
                max_abs_ref=float(np.abs(ref).max()) if ref.size else 0.0,
                rel_fro=float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got - ref)))


def check_rows(got, ref, floor, name, rtol=GRAD_RTOL, quiet=False):
    """Asserts the per-row bound for every row and the whole-matrix bound; returns the summary."""
    r = row_errors(got, ref, floor, rtol)
    if not quiet:
        print(f"        {name}: rows={len(r['err'])} relF={r['rel_fro']:.2e} max|diff|={r['max_abs']:.3e} "
              f"(max|ref|={r['max_abs_ref']:.3e}) worst row {r['worst_row']}: {r['worst_ratio']:.2f} of its allowance",
              flush=True)
    assert r["n_bad"] == 0, (f"{name}: {r['n_bad']} rows beyond their allowance, worst row {r['worst_row']} at "
                             f"{r['worst_ratio']:.2f}x (error {r['err'][r['worst_row']]:.3e}, "
                             f"allowed {r['tol'][r['worst_row']]:.3e})")
    assert r["rel_fro"] <= rtol, f"{name}: relative Frobenius error {r['rel_fro']:.3e}"
    return r


def check_step_grads(out_dX, out_dW, ref, W_A, X, tpos, scale, grad_scale, tag=""):
    """dX [B, D] and dW_A [A, D] of one step against the oracle's result `ref` (dict with dX, dWA, lse)."""
    B = X.shape[0]
    f_dx, f_dw = grad_floors(W_A, X, np.asarray(tpos), ref["lse"], scale, grad_scale / B)
    rx = check_rows(out_dX, ref["dX"], f_dx, f"{tag} dX")
    rw = check_rows(out_dW, ref["dWA"], f_dw, f"{tag} dW_A")
    return rx, rw
