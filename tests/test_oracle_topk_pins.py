"""Pins of the top-k oracle (Section 3.3.2: layer-wise top-k selection by divide and conquer) against things other
than itself: a stable library argsort, closed forms, brute force on tiny inputs, and the method's own claim that the
two-step selection is exact for every number of chunks."""
from __future__ import annotations

import numpy as np
import pytest

import synth


def _argsort_topk(g, k):
    # library routine: a stable sort of -|g| keeps equal magnitudes in ascending index
    order = np.argsort(-np.abs(g.astype(np.float64)), kind="stable")[:k]
    return order.astype(np.int32), g[order]


@pytest.mark.parametrize("n,k,seed", [(1, 1, 0), (7, 3, 1), (1000, 10, 2), (4097, 257, 3), (50_000, 50, 4), (3000, 3000, 5)])
def test_topk_matches_stable_argsort(orc, n, k, seed):
    g = (synth.normal(seed, synth.TID_GRAD_SET, 0, n) * 1e-3).astype(np.float32)
    if n > 100:  # plant ties: repeated values with both signs, and a run of zeros
        g[10:40] = np.float32(0.5) * np.where(np.arange(30) % 2 == 0, 1, -1)
        g[50:60] = 0.0
    idx, val = orc.topk_abs(g, k)
    ridx, rval = _argsort_topk(g, k)
    assert (idx == ridx).all() and (val.view(np.uint32) == rval.view(np.uint32)).all()


def test_topk_closed_forms(orc):
    n, k = 1001, 17
    ramp = (np.arange(1, n + 1) * np.where(np.arange(n) % 2 == 0, 1.0, -1.0)).astype(np.float32)  # |g_i| = i + 1
    idx, val = orc.topk_abs(ramp, k)
    assert idx.tolist() == list(range(n - 1, n - 1 - k, -1)) and (np.abs(val) == np.arange(n, n - k, -1)).all()
    assert (np.sign(val) == np.where(idx % 2 == 0, 1.0, -1.0)).all()  # the signed values come back
    # a constant tensor: the first k indices, in order; signed zeros are equal magnitudes
    idx, _ = orc.topk_abs(np.full(n, -2.5, dtype=np.float32), k)
    assert idx.tolist() == list(range(k))
    z = np.zeros(64, dtype=np.float32)
    z[1::2] = -0.0
    idx, val = orc.topk_abs(z, 5)
    assert idx.tolist() == [0, 1, 2, 3, 4] and np.signbit(val).tolist() == [False, True, False, True, False]
    # one large element among zeros, at the end; infinities beat every finite value
    z[63] = -1e-30
    z[7] = np.inf
    idx, val = orc.topk_abs(z, 3)
    assert idx.tolist() == [7, 63, 0] and val[1] == np.float32(-1e-30)
    # a subnormal is larger than zero
    z[:] = 0.0
    z[40] = np.float32(1e-45)
    assert orc.topk_abs(z, 1)[0].tolist() == [40]


@pytest.mark.parametrize("seed", range(6))
def test_topk_brute_force_repeated_maximum(orc, seed):
    rng = np.random.default_rng(seed)
    n, k = int(rng.integers(1, 40)), 0
    k = int(rng.integers(1, n + 1))
    g = rng.integers(-4, 5, size=n).astype(np.float32)  # small integers: many ties
    left, want = list(range(n)), []
    for _ in range(k):
        best = left[0]
        for i in left:  # strict comparison keeps the lowest index among equals
            if abs(float(g[i])) > abs(float(g[best])):
                best = i
        want.append(best)
        left.remove(best)
    idx, val = orc.topk_abs(g, k)
    assert idx.tolist() == want and (val == g[want]).all()


@pytest.mark.parametrize("n,k", [(10_000, 10), (10_000, 700), (12_345, 100), (513, 512), (64, 64)])
def test_two_step_selection_is_exact_for_every_chunk_count(orc, n, k):
    g = (synth.normal(9, synth.TID_GRAD_SET, 0, n) * 1e-2).astype(np.float32)
    g[n // 3:n // 3 + n // 10] = 0.0
    g[: n // 20] = np.round(g[: n // 20] * 400) / 400  # repeated magnitudes
    ref_idx, ref_val = orc.topk_abs(g, k)
    for M in (1, 2, 3, 7, 32, 100, n // 2, n):
        if M < 1 or M > n:
            continue
        idx, val = orc.topk_dc(g, k, M)
        assert (idx == ref_idx).all() and (val.view(np.uint32) == ref_val.view(np.uint32)).all(), M
    # a planted mistake would show: taking fewer than k per chunk is NOT exact (here all large values sit in one chunk)
    h = np.zeros(1000, dtype=np.float32)
    h[:20] = np.arange(20, 0, -1)
    idx, _ = orc.topk_dc(h, 20, 10)
    assert idx.tolist() == list(range(20))


def test_group_of_tensors_is_tensor_by_tensor(orc):
    sizes = [5, 64, 1000, 1, 4096, 333]
    g, offs = synth.grad_tensor_set(3, sizes, zero_every=2)
    k = np.array([2, 64, 10, 1, 5, 33], dtype=np.int32)
    idx, val = orc.topk_group(g, offs, k)
    idx2, val2 = orc.topk_group(g, offs, k, M=np.array([1, 4, 7, 1, 32, 5], dtype=np.int32))
    assert (idx == idx2).all() and (val.view(np.uint32) == val2.view(np.uint32)).all()
    o = 0
    for t, n in enumerate(sizes):
        ridx, rval = _argsort_topk(g[offs[t]:offs[t + 1]], int(k[t]))
        assert (idx[o:o + k[t]] == ridx).all() and (val[o:o + k[t]] == rval).all()
        o += int(k[t])


def test_resnet50_sizes_add_up():
    sizes = synth.resnet50_tensor_sizes()
    # the parameter count of the architecture as published: 25,557,032 in 161 tensors
    assert len(sizes) == 161 and sum(sizes) == 25_557_032 and max(sizes) == 512 * 512 * 9
    k = synth.topk_counts(sizes)
    assert k.min() == 1 and k.max() == 2359
