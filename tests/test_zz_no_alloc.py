"""knn_select_active_static (the selection for callers that cannot allocate: its scratch memory is a static device
array inside the library) against knn_select_active, through the C ABI: two calls in a row, the second with a
smaller input, every output bit for bit; then the table path of large class counts, and a repeat of the first
call (the array keeps the previous call's contents)."""
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


def _both(ks, C, K, B, M, seed, empty=0.0):
    print(f"[no-alloc] C={C} K={K} B={B} M={M} seed={seed}", flush=True)
    G = dev(synth.graph_synthetic(seed, C, K, locality=4, empty_frac=empty))
    y = dev(synth.labels_uniform(seed, B, C))
    # outputs of the static call are allocated up front: the call itself gets nothing but pointers
    out = (torch.full((M,), -7, dtype=torch.int32, device="cuda"), torch.full((1,), -7, dtype=torch.int32, device="cuda"),
           torch.full((B,), -7, dtype=torch.int32, device="cuda"))
    st = torch.zeros(1, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    a1, n1, t1, s1 = ks.knn_select_active_static(y, G, C, M, out=out, dev_status=st)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    a0, n0, t0, s0 = ks.knn_select_active(y, G, C, M)
    torch.cuda.synchronize()
    assert int(s0.item()) == 0 and int(s1.item()) == 0
    assert torch.equal(n0, n1) and torch.equal(a0, a1) and torch.equal(t0, t1)
    return int(n1.item())


def test_static_selection_equals_the_workspace_one_on_two_calls_in_a_row(ks):
    n_big = _both(ks, 390_625, 32, 1_024, 32_768, 0)            # the headline shape
    n_small = _both(ks, 3_000, 16, 128, 600, 2, empty=0.3)      # a smaller input right after it
    assert n_big > n_small > 0
    _both(ks, 100_000, 16, 256, 4_096, 0)                       # the cut bites
    _both(ks, 450_000, 8, 300, 2_000, 3)                        # above the bitmap path's limit: the table path
    assert _both(ks, 390_625, 32, 1_024, 32_768, 0) == n_big    # and the first one again


def test_static_selection_rejects_what_does_not_fit(ks):
    y = dev(synth.labels_uniform(0, 2_048, 1_000_000))
    G = dev(synth.graph_synthetic(0, 1_000_000, 64))
    with pytest.raises(ks.KsError) as e:
        ks.knn_select_active_static(y, G, 1_000_000, 131_072)
    assert e.value.code == ks.KS_UNSUPPORTED
