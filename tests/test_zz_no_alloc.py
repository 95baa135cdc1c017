"""ann_search_static (temporaries in the library's static device array, no allocation) against
ann_search, through the C ABI: same bytes out, on calls in a row that reuse the array."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def clustered_u8(rng, n, n_centres):
    cen = rng.integers(30, 226, (n_centres, 128)).astype(np.float64)
    lab = np.sort(rng.integers(0, n_centres, n))
    x = np.clip(np.rint(cen[lab] + rng.standard_normal((n, 128)) * 14.0), 0, 255).astype(np.uint8)
    off = np.searchsorted(lab, np.arange(n_centres + 1)).astype(np.int64)
    return x, cen.astype(np.uint8), off


def test_static_scratch_search_equals_ann_search_on_consecutive_calls():
    import torch

    from paper_2512_02278_amd import ann

    if not torch.cuda.is_available():
        pytest.fail("needs the MI355X")
    L = ann.lib()
    rng = np.random.default_rng(123)
    x, cen, off = clustered_u8(rng, 30_000, 40)
    g = rng.integers(0, 30_000, (30_000, 32)).astype(np.int32)
    for c in range(40):  # edges stay inside a cluster, as in the workloads
        lo, hi = int(off[c]), int(off[c + 1])
        g[lo:hi] = rng.integers(lo, hi, (hi - lo, 32))
    dev = "cuda:0"
    xt, gt = torch.from_numpy(x).to(dev), torch.from_numpy(g).to(dev)
    ct, ot = torch.from_numpy(cen).to(dev), torch.from_numpy(off).to(dev)
    h = ann.ann_index_load(xt, gt, n_entry=32, entry_mode=ann.ANN_ENTRY_ROUTED, seed=11, centroids=ct, cluster_offsets=ot,
                           route_c=2)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    # a batch that runs grouped by cluster, then smaller ones (routing partials; a batch below one workgroup)
    for nq in (20_000, 3_000, 17, 20_000):
        q = torch.from_numpy(x[rng.integers(0, 30_000, nq)]).to(dev)
        want_i = torch.empty((nq, 10), dtype=torch.int32, device=dev)
        want_d = torch.empty((nq, 10), dtype=torch.int32, device=dev)
        got_i, got_d = torch.full_like(want_i, -7), torch.full_like(want_d, -7)
        assert L.ann_search(h.ptr, q.data_ptr(), nq, 10, 64, 2, 60, want_i.data_ptr(), want_d.data_ptr(), stream) == ann.ANN_OK
        torch.cuda.synchronize()
        assert L.ann_search_static(h.ptr, q.data_ptr(), nq, 10, 64, 2, 60, got_i.data_ptr(), got_d.data_ptr(), stream) == ann.ANN_OK, ann.ann_last_error()
        torch.cuda.synchronize()
        assert torch.equal(got_i, want_i) and torch.equal(got_d, want_d), nq
        assert int((got_i >= 0).sum()) > 0
    # beyond the limit: an error, nothing launched, outputs untouched
    nq_big = ann.ANN_STATIC_SCRATCH_BYTES // 8
    got_i.fill_(-7)
    rc = L.ann_search_static(h.ptr, q.data_ptr(), nq_big, 10, 64, 2, 60, got_i.data_ptr(), got_d.data_ptr(), stream)
    torch.cuda.synchronize()
    assert rc == ann.ANN_EUNSUPPORTED and "static scratch" in ann.ann_last_error()
    assert int((got_i != -7).sum()) == 0
    ann.ann_free(h)

    # an index with uniform entries needs no temporaries
    h = ann.ann_index_load(xt, gt, n_entry=32, seed=11)
    q = torch.from_numpy(x[:500]).to(dev)
    want = ann.ann_search(h, q, 10, 64, 2, 60)
    got = ann.ann_search_static(h, q, 10, 64, 2, 60, torch.empty_like(want[0]), torch.empty_like(want[1]))
    torch.cuda.synchronize()
    assert torch.equal(got[0], want[0]) and torch.equal(got[1], want[1])
    ann.ann_free(h)
