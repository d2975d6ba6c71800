"""lorann_search_noalloc (the entry point for callers that cannot allocate) against lorann_search_async, through the
C ABI: same kernels, buffers carved from the GPU's fixed scratch region instead of allocated ones, so the results must
be bit-identical.  Collected last on purpose (see the file name)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2410_18926_amd import binding
    assert binding.LIB_PATH.exists(), "build the HIP library first (python -m paper_2410_18926_amd.build)"
    assert torch.cuda.is_available(), "these tests need the GPU"
    return binding


def _random_index(rng, n, d, L, r, metric, dp):
    cuts = np.sort(rng.choice(np.arange(1, n), size=L - 1, replace=False))
    off = np.concatenate([[0], cuts, [n]]).astype(np.int64)
    corpus = rng.normal(size=(n, d)).astype(np.float32)
    if metric == 2:
        corpus /= np.linalg.norm(corpus, axis=1, keepdims=True)
    P = None if dp == d else np.linalg.qr(rng.normal(size=(d, d)))[0][:, :dp].astype(np.float32)
    return dict(metric=metric, n=n, d=d, dp=dp, r=r, L=L, centroids=rng.normal(size=(L, dp)).astype(np.float32), P=P,
                A=rng.integers(-127, 128, size=(L, r, dp)).astype(np.int8), B=rng.integers(-127, 128, size=(n, r)).astype(np.int8),
                scale_A=rng.uniform(0.01, 0.1, L).astype(np.float32), scale_B=rng.uniform(0.01, 0.1, L).astype(np.float32),
                cluster_offsets=off, corpus=corpus, ids=rng.permutation(n).astype(np.int64))


@pytest.mark.parametrize("metric", [0, 1, 2])
def test_two_calls_in_a_row_match_the_allocating_entry_point(B, metric):
    """A first call, then a second one with a smaller batch and other w, m (every buffer moves inside the region and
    finds the first call's contents there): both bit-identical to lorann_search_async on the same inputs.  The calls
    are made BEFORE the index has ever allocated a workspace, and the free device memory does not change."""
    rng = np.random.default_rng(300 + metric)
    ix = _random_index(rng, n=6000, d=72, L=40, r=24, metric=metric, dp=48)
    dev = torch.device("cuda:0")
    q1 = torch.from_numpy(rng.normal(size=(700, 72)).astype(np.float32)).to(dev)
    q2 = torch.from_numpy(rng.normal(size=(90, 72)).astype(np.float32)).to(dev)
    calls = [(q1, 10, 6, 80), (q2, 7, 9, 33)]
    outs = [(torch.full((q.shape[0], k), -7, dtype=torch.int64, device=dev), torch.full((q.shape[0], k), -7.0, dtype=torch.float32, device=dev))
            for q, k, w, m in calls]
    # (a first index takes whatever the runtime itself sets up on the first launch of a kernel out of the measurement)
    warm = B.Index(**ix)
    warm.search_noalloc(q1, 10, 6, 80, out=(torch.empty_like(outs[0][0]), torch.empty_like(outs[0][1])))
    warm.search_noalloc(q2, 7, 9, 33, out=(torch.empty_like(outs[1][0]), torch.empty_like(outs[1][1])))
    torch.cuda.synchronize()
    warm.close()
    gix = B.Index(**ix)
    gix.use_torch_stream()
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    for (q, k, w, m), o in zip(calls, outs):
        gix.search_noalloc(q, k, w, m, out=o)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free0, "the non-allocating entry point changed the free device memory"
    for (q, k, w, m), o in zip(calls, outs):
        a_ids, a_d = gix.search(q, k, w, m, asynchronous=True)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(o[0].cpu().numpy(), a_ids.cpu().numpy())
        np.testing.assert_array_equal(o[1].cpu().numpy(), a_d.cpu().numpy())
        assert (o[0] != -7).any()
    # once more after the allocating path has run, in the opposite order
    for (q, k, w, m), o in reversed(list(zip(calls, outs))):
        n_ids, n_d = gix.search_noalloc(q, k, w, m, out=(torch.empty_like(o[0]), torch.empty_like(o[1])))
        torch.cuda.synchronize()
        np.testing.assert_array_equal(n_ids.cpu().numpy(), o[0].cpu().numpy())
        np.testing.assert_array_equal(n_d.cpu().numpy(), o[1].cpu().numpy())
    gix.close()


def test_sizes_beyond_the_region_and_other_refusals(B):
    rng = np.random.default_rng(77)
    ix = _random_index(rng, n=5000, d=32, L=300, r=8, metric=0, dp=32)
    dev = torch.device("cuda:0")
    gix = B.Index(**ix)
    big = torch.zeros((30000, 32), dtype=torch.float32, device=dev)       # 30000 x 300 approximate scores alone are 36 MB
    ids = torch.full((30000, 5), -7, dtype=torch.int64, device=dev)
    d = torch.full((30000, 5), -7.0, dtype=torch.float32, device=dev)
    with pytest.raises(B.LorannError) as ei:
        gix.search_noalloc(big, 5, 4, 20, out=(ids, d))
    assert ei.value.code == B.LORANN_E_UNSUPPORTED and "bytes of workspace" in str(ei.value)
    torch.cuda.synchronize()
    assert (ids == -7).all() and (d == -7.0).all()                        # refused before anything was enqueued
    gix.profile_enable(True)
    with pytest.raises(B.LorannError) as ei:
        gix.search_noalloc(big[:10], 5, 4, 20, out=(ids[:10], d[:10]))
    assert ei.value.code == B.LORANN_E_INVAL
    gix.profile_enable(False)
    # the ordinary argument checks still apply, and a small call after the refusals works
    with pytest.raises(B.LorannError):
        gix.search_noalloc(big[:10], 5, 400, 20, out=(ids[:10], d[:10]))
    q = torch.from_numpy(rng.normal(size=(10, 32)).astype(np.float32)).to(dev)
    gix.search_noalloc(q, 5, 4, 20, out=(ids[:10], d[:10]))
    s_ids, s_d = gix.search(q, 5, 4, 20)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(ids[:10].cpu().numpy(), s_ids.cpu().numpy())
    np.testing.assert_array_equal(d[:10].cpu().numpy(), s_d.cpu().numpy())
    gix.close()
