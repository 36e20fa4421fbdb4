"""GPU parity of the layer-wise top-k selection (Section 3.3.2: divide-and-conquer top-k, grouped tensors): indices and
values are compared bit for bit with the CPU oracle's definition (a full sort), over sizes that span one to many chunks
with ragged tails, every path of the workgroup routine (the histogram bin fits; refinement by the lower bits; more equal
magnitudes than the sort array holds), forced chunk counts (the paper's two steps and deeper trees), the sampled path of
large tensors with samples that mislead in both directions, and the full gradient set of a ResNet-50."""
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


def run(ks, g, offs, k, chunks=0):
    plan = ks.grad_topk_plan(offs, k, chunks)
    gd = torch.from_numpy(g).cuda()
    idx, val = ks.grad_topk_select(gd, plan)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), val.cpu().numpy(), plan


def check(ks, orc, g, offs, k, chunks=0):
    idx, val, plan = run(ks, g, offs, k, chunks)
    eidx, eval_ = orc.topk_group(g, offs, k)
    assert np.array_equal(idx, eidx), f"indices differ (chunks={chunks}, M={plan.chunks()[:8]})"
    assert np.array_equal(val.view(np.uint32), eval_.view(np.uint32))
    return plan


def one(g):
    return np.ascontiguousarray(g, dtype=np.float32), np.array([0, g.size], dtype=np.int64)


@pytest.mark.parametrize("n,k", [(1, 1), (5, 5), (5, 2), (1000, 10), (8192, 64), (8193, 8), (100_003, 100), (1_000_000, 1000),
                                 (300_000, 4096), (4096, 4096), (20_000, 4000)])
@pytest.mark.parametrize("chunks", [0, 1, 3, 64])
def test_single_tensor_matches_oracle(ks, orc, n, k, chunks):
    g = (synth.normal(n + k, synth.TID_GRAD_SET, 0, n) * 1e-3).astype(np.float32)
    if n >= 1000:  # ties with both signs, a run of zeros
        g[100:160] = np.float32(0.25) * np.where(np.arange(60) % 2 == 0, 1, -1)
        g[n // 2:n // 2 + n // 10] = 0.0
    print(f"case n={n} k={k} chunks={chunks}", flush=True)
    check(ks, orc, *one(g), np.array([k], dtype=np.int32), chunks)


def test_values_in_one_histogram_bin_are_refined_by_the_lower_bits(ks, orc):
    # all magnitudes in [1, 1.0001): one bin of the first pass holds everything, far more than the sort array
    n = 300_000
    g = (1.0 + 1e-4 * synth.uniform01(1, synth.TID_GRAD_SET, 0, n)).astype(np.float32)
    g[::3] *= -1
    for k in (1, 77, 4096):
        for chunks in (0, 1, 5):
            print(f"case narrow k={k} chunks={chunks}", flush=True)
            check(ks, orc, *one(g), np.array([k], dtype=np.int32), chunks)


def test_more_equal_magnitudes_than_the_sort_array_holds(ks, orc):
    n = 200_000
    const = np.full(n, -3.0, dtype=np.float32)
    zeros = np.zeros(n, dtype=np.float32)
    zeros[1::2] = -0.0
    zeros[[7, 150_000, 199_999]] = [1e-20, -2e-20, 3e-20]  # k beyond the non-zeros: the rest are zeros by index
    steps = np.round(synth.normal(2, synth.TID_GRAD_SET, 0, n) * 2).astype(np.float32)  # a handful of distinct values
    for name, g in (("const", const), ("zeros", zeros), ("steps", steps)):
        for k in (1, 10, 4096):
            for chunks in (0, 1, 4):
                print(f"case {name} k={k} chunks={chunks}", flush=True)
                check(ks, orc, *one(g), np.array([k], dtype=np.int32), chunks)


def test_non_finite_values_rank_by_their_bit_patterns(ks, orc):
    n = 50_000
    g = (synth.normal(3, synth.TID_GRAD_SET, 0, n)).astype(np.float32)
    g[[5, 40_000]] = [np.inf, -np.inf]
    g[[17, 30_000]] = np.nan
    idx, val, _ = run(ks, *one(g), np.array([6], dtype=np.int32))
    assert sorted(idx[:2].tolist()) == [17, 30_000] and idx[2:4].tolist() == [5, 40_000]
    check(ks, orc, *one(g), np.array([6], dtype=np.int32))


def test_group_of_tensors_and_independence_of_the_chunk_count(ks, orc):
    sizes = [1, 7, 64, 1000, 8192, 8193, 40_000, 123_457, 600_000, 3, 2_000_000]
    g, offs = synth.grad_tensor_set(4, sizes, zero_every=2)
    k = np.array([1, 7, 3, 10, 8, 100, 40, 1234, 600, 1, 2000], dtype=np.int32)
    base = None
    for chunks in (0, 1, 2, 37):
        print(f"case group chunks={chunks}", flush=True)
        check(ks, orc, g, offs, k, chunks)
        idx, val, _ = run(ks, g, offs, k, chunks)
        if base is None:
            base = (idx, val)
        assert np.array_equal(idx, base[0]) and np.array_equal(val.view(np.uint32), base[1].view(np.uint32))


def test_sampled_path_and_what_happens_when_the_sample_misleads(ks, orc):
    """Tensors of several chunks take a threshold from 4,096 evenly spaced elements; the chunks then hand on what lies at
    or above it and a final step selects.  The count that arrives is checked, so a sample that misleads costs time, not
    correctness: here (a) gradient-like values, the path as planned; (b) all large values sit exactly on sampled
    positions, so the threshold is far too high and fewer than k items arrive; (c) all large values sit between the
    sampled positions and everything else is equal, so the threshold is the common value and every element passes;
    (d) a tensor beside them that keeps its own path.  Bit-exact against the oracle in every case."""
    n, k = 600_000, 600
    pos = (np.arange(4096, dtype=np.int64) * n) // 4096
    base = (synth.normal(21, synth.TID_GRAD_SET, 0, n) * 1e-3).astype(np.float32)
    on_sample = (base * 1e-3).astype(np.float32)
    on_sample[pos[::8]] = (1.0 + synth.uniform01(22, synth.TID_GRAD_SET, 0, 512)).astype(np.float32)   # 512 large values < k
    off_sample = np.full(n, 0.5, dtype=np.float32)
    between = np.setdiff1d(np.arange(n), pos)[::200][:2000]
    off_sample[between] = (2.0 + synth.uniform01(23, synth.TID_GRAD_SET, 0, between.size)).astype(np.float32)
    for name, g in (("gradient-like", base), ("large values on the sample", on_sample), ("large values off the sample", off_sample)):
        print(f"case sampled path: {name}", flush=True)
        plan = check(ks, orc, *one(g), np.array([k], dtype=np.int32))
        assert plan.steps() == [3]
    g_all = np.concatenate([base, on_sample, off_sample, base[:50_000]])
    offs = np.array([0, n, 2 * n, 3 * n, 3 * n + 50_000], dtype=np.int64)
    print("case sampled path: all of them in one group", flush=True)
    check(ks, orc, g_all, offs, np.array([k, k, 2000, 50], dtype=np.int32))


def test_resnet50_gradient_set(ks, orc):
    sizes = synth.resnet50_tensor_sizes()
    g, offs = synth.grad_tensor_set(0, sizes)
    k = synth.topk_counts(sizes)
    print("case resnet50 set", flush=True)
    plan = check(ks, orc, g, offs, k)
    assert max(plan.chunks()) >= 30 and plan.n_out == int(k.sum())
    # a second call on the same buffers gives the same bits (nothing is left over in the workspace that matters)
    gd = torch.from_numpy(g).cuda()
    ws = torch.empty(plan.ws_bytes, dtype=torch.uint8, device="cuda")
    a = ks.grad_topk_select(gd, plan, ws=ws)
    a = (a[0].clone(), a[1].clone())
    ws.fill_(0xFF)
    b = ks.grad_topk_select(gd, plan, ws=ws)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
