"""Parity of the HIP library against the CPU oracle on the same seeded inputs (needs an MI355X).

Bars: integer stages (query codes, selected clusters, re-quantized vectors, int32 score accumulators,
candidate sets) bit-exact; combined scales bit-exact (same double expression); re-rank distances within 1e-4
relative; returned ids identical except at distance ties within 1e-5.
"""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from tests.parity_util import assert_topk_equal, oracle_distance_of, rounding_abs_tol, y_offsets

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2410_18926_amd import binding
    assert binding.LIB_PATH.exists(), "build the HIP library first (python -m paper_2410_18926_amd.build)"
    assert torch.cuda.is_available(), "these tests need the GPU"
    return binding


def _stagewise(B, wl, ix, queries, k=None, w=None, m=None, device_inputs=True):
    a = ix.numpy()
    k, w, m = k or wl.k, w or wl.w, m or wl.m
    oix = O.OracleIndex(a)
    o_ids, o_d, ost = O.search(oix, queries, k, w, m, stages=True)
    src = ix.to("cuda") if device_inputs else ix.to("cpu")
    gix = B.Index.from_arrays(src)
    yo = y_offsets(ost["sel"], a["cluster_offsets"])
    q_in = torch.from_numpy(queries).cuda() if device_inputs else queries
    g_ids, g_d, gst = gix.search_stages(q_in, k, w, m, y_off=yo)
    tag = wl.name
    np.testing.assert_array_equal(gst["qproj"], ost["qproj"], err_msg=f"{tag}: projected queries")
    np.testing.assert_array_equal(gst["q8"], ost["q8"], err_msg=f"{tag}: query codes")
    np.testing.assert_array_equal(gst["dx"], ost["dx"], err_msg=f"{tag}: query step sizes")
    np.testing.assert_array_equal(gst["sel"], ost["sel"], err_msg=f"{tag}: selected clusters")
    np.testing.assert_array_equal(gst["z"], ost["z"], err_msg=f"{tag}: re-quantized vectors")
    np.testing.assert_array_equal(gst["sigma"], ost["sigma"], err_msg=f"{tag}: pair scales")
    np.testing.assert_array_equal(gst["rho0"], ost["rho0"], err_msg=f"{tag}: unquantized first components")
    # int32 score accumulators of every point of every selected cluster
    nq = queries.shape[0]
    y_ref = np.empty_like(gst["y"])
    for s in range(nq * w):
        qi, j = divmod(s, w)
        c = int(ost["sel"][qi, j])
        o0, o1 = int(a["cluster_offsets"][c]), int(a["cluster_offsets"][c + 1])
        y_ref[yo[s]:yo[s + 1]] = O.pair_accumulators(ost["z"][qi, j], a["B"][o0:o1])
    np.testing.assert_array_equal(gst["y"], y_ref, err_msg=f"{tag}: int32 score accumulators (matrix-core kernel)")
    # best estimated score of every pair, as the batched matrix-core kernel found it (it only prunes, so a wrong
    # value would not show in the candidates): equal to the maximum of the oracle's step-5 scores
    np.testing.assert_array_equal(gst["pmax"], ost["pair_best"], err_msg=f"{tag}: per-pair best scores")
    # candidate sets (the library returns them unordered)
    np.testing.assert_array_equal(np.sort(gst["cand_rows"].astype(np.int64), axis=1), np.sort(ost["cand_rows"], axis=1),
                                  err_msg=f"{tag}: candidate sets")
    n_tie = assert_topk_equal(g_ids, g_d, o_ids, o_d, tag, abs_tol=rounding_abs_tol(queries, a["corpus"], a["metric"]),
                              exact=oracle_distance_of(a, queries))
    # the exact per-query selection kernel (the fallback of the batched path) must give the same candidates
    gix.set_exact_selection(True)
    e_ids, e_d, est = gix.search_stages(q_in, k, w, m, y_off=yo)
    gix.set_exact_selection(False)
    np.testing.assert_array_equal(est["y"], y_ref, err_msg=f"{tag}: int32 score accumulators (per-query kernel)")
    np.testing.assert_array_equal(np.sort(est["cand_rows"].astype(np.int64), axis=1), np.sort(ost["cand_rows"], axis=1),
                                  err_msg=f"{tag}: candidate sets (per-query kernel)")
    np.testing.assert_array_equal(e_ids, g_ids)
    np.testing.assert_array_equal(e_d, g_d)
    # plain entry point returns the same as the staged one; second call is bitwise identical (determinism)
    p_ids, p_d = gix.search(q_in, k, w, m)
    p_ids2, p_d2 = gix.search(q_in, k, w, m)
    if device_inputs:
        p_ids, p_d, p_ids2, p_d2 = (t.cpu().numpy() for t in (p_ids, p_d, p_ids2, p_d2))
    np.testing.assert_array_equal(p_ids, g_ids)
    np.testing.assert_array_equal(p_d, g_d)
    np.testing.assert_array_equal(p_ids2, p_ids)
    np.testing.assert_array_equal(p_d2, p_d)
    if nq <= 64:
        # batches of up to 64 queries take the query-major path (no bucketing); the same queries three times over
        # form a batch that takes the cluster-batched path: every copy must come out the same
        reps = 64 // nq + 1
        t_in = torch.from_numpy(np.tile(queries, (reps, 1))).cuda() if device_inputs else np.tile(queries, (reps, 1))
        t_ids, t_d, tst = gix.search_stages(t_in, k, w, m)
        for rep in range(reps):
            sl = slice(rep * nq, (rep + 1) * nq)
            np.testing.assert_array_equal(t_ids[sl], g_ids, err_msg=f"{tag}: cluster-batched path, copy {rep}")
            np.testing.assert_array_equal(t_d[sl], g_d)
            np.testing.assert_array_equal(tst["z"][sl], gst["z"])
            np.testing.assert_array_equal(tst["sigma"][sl], gst["sigma"])
            np.testing.assert_array_equal(tst["pmax"][sl], gst["pmax"])
            np.testing.assert_array_equal(np.sort(tst["cand_rows"][sl], axis=1), np.sort(gst["cand_rows"], axis=1))
    gix.close()
    return n_tie


def test_small_workloads_stagewise(B, small_indexes):
    """Four small configurations: Euclidean without projection, inner product and cosine with projection
    (d not a multiple of the tile sizes, ragged clusters), heavy-tailed norms."""
    for name, (wl, ix, corpus, queries) in small_indexes.items():
        _stagewise(B, wl, ix, queries)


def test_small_workloads_host_pointers(B, small_indexes):
    wl, ix, corpus, queries = small_indexes["cos_P"]
    _stagewise(B, wl, ix, queries, device_inputs=False)


def test_tiny_config_stagewise(B):
    """The smallest configured workload (20 000 x 128, 64 clusters, r = 32, w = 8, m = 100, Euclidean), all 1000 queries."""
    from paper_2410_18926_amd.synth import get_workload, make_dataset, build_index
    wl = get_workload("tiny")
    corpus, queries = make_dataset(wl)
    ix = build_index(corpus, wl)
    _stagewise(B, wl, ix, queries.numpy())


@pytest.mark.parametrize("r,dp,d", [(8, 16, 30), (24, 48, 48), (48, 64, 100), (64, 128, 128), (16, 1024, 1024)])
def test_rank_and_dimension_variants(B, r, dp, d):
    """Ranks that need K padding on the matrix cores (24, 48), minimum and maximum d', d not a multiple of 4."""
    from paper_2410_18926_amd.synth import make_dataset, build_index
    from paper_2410_18926_amd.synth.workloads import Workload, IP
    wl = Workload(f"v-r{r}-dp{dp}", 70 + r, n=1500, d=d, nq=33, G=6, alpha=1.0, normalize=True, lognormal_norms=None,
                  metric=IP, L=7, dp=dp, r=r, w=3, m=37, n_train=800, w_train=3)
    corpus, queries = make_dataset(wl)
    ix = build_index(corpus, wl)
    _stagewise(B, wl, ix, queries.numpy())


@pytest.mark.parametrize("metric", [0, 1, 2])
@pytest.mark.parametrize("r", [32, 48])
@pytest.mark.parametrize("dense", [False, True])
def test_matrix_core_scores_per_pair_maxima_and_accumulators(B, metric, r, dense):
    """The second 8-bit product on the matrix cores, compared directly: every int32 accumulator it forms and the best
    score it reports for every (query, cluster) pair, bit for bit against the oracle's step 5 - in both launch shapes
    (dense: work items of 64 pairs x 512 points on a persistent grid; else one wavefront streams a cluster), with one
    and two k-steps (r = 32, 48), for the three metrics, on cluster sizes that end inside the first 32-point tile of
    a pair of tiles, inside the second, and on a boundary, with empty clusters, and with scores that are all
    negative (so that anything read beyond a cluster's end - zeros - would win the maximum)."""
    rng = np.random.default_rng(40 + 7 * metric + r + (1 if dense else 0))
    sizes = [1, 31, 32, 33, 63, 64, 65, 95, 96, 97, 0, 700, 1024, 1025, 1056, 1057, 0, 130]
    L, d = len(sizes), 32
    n = sum(sizes)
    ix = _random_index(rng, n=n, d=d, L=L, r=r, metric=metric)
    off = np.zeros(L + 1, np.int64)
    np.cumsum(sizes, out=off[1:])
    ix["cluster_offsets"] = off
    nq = 400 if dense else 12
    w, m, k = L, 50, 5
    q = rng.normal(size=(nq, d)).astype(np.float32)
    for variant in ("random", "negative"):
        if variant == "negative":
            # Euclidean only: large row norms make every score negative (for inner products the clusters of one
            # point already give negative maxima about half of the time)
            if metric != 1:
                continue
            ix = dict(ix)
            ix["corpus"] = (ix["corpus"] * 50.0).astype(np.float32)
        oix = O.OracleIndex(ix)
        o_ids, o_d, ost = O.search(oix, q, k, w, m, stages=True)
        yo = y_offsets(ost["sel"], off)
        gix = B.Index(**ix)
        g_ids, g_d, gst = gix.search_stages(q, k, w, m, y_off=yo)
        gix.close()
        np.testing.assert_array_equal(gst["sel"], ost["sel"])
        np.testing.assert_array_equal(gst["z"], ost["z"])
        y_ref = np.empty_like(gst["y"])
        for s_ in range(nq * w):
            qi, j = divmod(s_, w)
            c = int(ost["sel"][qi, j])
            y_ref[yo[s_]:yo[s_ + 1]] = O.pair_accumulators(ost["z"][qi, j], ix["B"][off[c]:off[c + 1]])
        np.testing.assert_array_equal(gst["y"], y_ref, err_msg=f"{variant}: int32 accumulators of the matrix-core kernel")
        np.testing.assert_array_equal(gst["pmax"], ost["pair_best"], err_msg=f"{variant}: per-pair best scores")
        assert np.isneginf(ost["pair_best"]).any()          # the empty clusters
        if variant == "negative":
            assert (ost["pair_best"][np.isfinite(ost["pair_best"])] < 0).all()
        np.testing.assert_array_equal(np.sort(gst["cand_rows"].astype(np.int64), axis=1), np.sort(ost["cand_rows"], axis=1))


def test_probe_everything_equals_exact_knn(B, small_indexes):
    """w = L and m = n: the library must return the exact k-NN (checked against the oracle's brute force)."""
    for name in ("l2_noP", "ip_P"):
        wl, ix, corpus, queries = small_indexes[name]
        a = ix.numpy()
        gix = B.Index.from_arrays(ix.to("cuda"))
        ids, d = gix.search(queries[:16], wl.k, wl.L, wl.n)
        e_ids, e_d = O.exact_knn(a["corpus"], queries[:16], wl.metric, wl.k, ids=a["ids"])
        assert_topk_equal(ids, d, e_ids, e_d, name)
        gix.close()


def test_edge_cases(B, small_indexes):
    wl, ix, corpus, queries = small_indexes["l2_P_norms"]
    a = ix.numpy()
    oix = O.OracleIndex(a)
    gix = B.Index.from_arrays(ix.to("cuda"))
    # empty batch
    ids, d = gix.search(np.zeros((0, wl.d), np.float32), 5, 2, 10)
    assert ids.shape == (0, 5)
    # single query, k == m, w == 1
    for (k, w, m) in [(1, 1, 1), (7, 1, 7), (10, wl.L, 4096), (3, 2, 3)]:
        o_ids, o_d = O.search(oix, queries[:3], k, w, m)
        g_ids, g_d = gix.search(queries[:3], k, w, m)
        assert_topk_equal(g_ids, g_d, o_ids, o_d, f"k={k} w={w} m={m}")
    # zero query: all codes zero, all scores equal -> candidates are the lowest rows of the selected clusters
    zq = np.zeros((2, wl.d), np.float32)
    o_ids, o_d = O.search(oix, zq, 5, 3, 20)
    g_ids, g_d = gix.search(zq, 5, 3, 20)
    assert_topk_equal(g_ids, g_d, o_ids, o_d, "zero query")
    # invalid arguments
    for (k, w, m, code) in [(0, 1, 1, -1), (5, 1, 4, -1), (1, 0, 1, -1), (1, wl.L + 1, 1, -1), (1, 1, 5000, -4)]:
        with pytest.raises(B.LorannError) as e:
            gix.search(queries[:2], k, w, m)
        assert e.value.code == code
    gix.close()


def test_empty_clusters_and_few_points(B):
    """Clusters without points, fewer scored points than m and than k (padding with -1 / +inf)."""
    rng = np.random.default_rng(5)
    d, L, r = 16, 5, 8
    corpus = rng.normal(size=(9, d)).astype(np.float32)
    ix = dict(metric=0, n=9, d=d, dp=d, r=r, L=L, centroids=rng.normal(size=(L, d)).astype(np.float32), P=None,
              A=rng.integers(-127, 128, size=(L, r, d)).astype(np.int8), B=rng.integers(-127, 128, size=(9, r)).astype(np.int8),
              scale_A=rng.uniform(0.01, 0.1, L).astype(np.float32), scale_B=rng.uniform(0.01, 0.1, L).astype(np.float32),
              cluster_offsets=np.array([0, 0, 4, 4, 4, 9], np.int64), corpus=corpus, ids=np.arange(100, 109, dtype=np.int64))
    q = rng.normal(size=(6, d)).astype(np.float32)
    gix = B.Index(**ix)
    oix = O.OracleIndex(ix)
    for (k, w, m) in [(4, 5, 30), (12, 5, 30), (3, 2, 5), (2, 1, 2)]:
        o_ids, o_d = O.search(oix, q, k, w, m)
        g_ids, g_d = gix.search(q, k, w, m)
        assert_topk_equal(g_ids, g_d, o_ids, o_d, f"k={k} w={w} m={m}")
    gix.close()


def test_score_ties_resolve_to_lower_rows(B):
    """Many equal estimated scores (duplicate codes): the candidate set must take the lower rows."""
    rng = np.random.default_rng(9)
    d, L, r, n = 16, 3, 8, 600
    corpus = rng.normal(size=(n, d)).astype(np.float32)
    codes = rng.integers(-3, 4, size=(n, r)).astype(np.int8)          # tiny alphabet => massive score ties
    ix = dict(metric=0, n=n, d=d, dp=d, r=r, L=L, centroids=rng.normal(size=(L, d)).astype(np.float32), P=None,
              A=rng.integers(-127, 128, size=(L, r, d)).astype(np.int8), B=codes,
              scale_A=np.full(L, 0.01, np.float32), scale_B=np.full(L, 0.02, np.float32),
              cluster_offsets=np.array([0, 250, 400, n], np.int64), corpus=corpus, ids=None)
    q = rng.normal(size=(20, d)).astype(np.float32)
    gix = B.Index(**ix)
    oix = O.OracleIndex(ix)
    o_ids, o_d, ost = O.search(oix, q, 10, 3, 64, stages=True)
    g_ids, g_d, gst = gix.search_stages(q, 10, 3, 64)
    np.testing.assert_array_equal(np.sort(gst["cand_rows"].astype(np.int64), axis=1), np.sort(ost["cand_rows"], axis=1))
    assert_topk_equal(g_ids, g_d, o_ids, o_d, "ties")
    gix.close()


def test_survivor_overflow_falls_back_to_exact_kernel(B):
    """All estimated scores equal: the bound equals that score, every point of the probed clusters survives the
    filter, the survivor lists overflow, and the exact per-query kernel must finish those queries - with the
    lowest rows as candidates."""
    rng = np.random.default_rng(11)
    d, L, r, n = 16, 4, 8, 9000
    corpus = rng.normal(size=(n, d)).astype(np.float32)
    ix = dict(metric=0, n=n, d=d, dp=d, r=r, L=L, centroids=rng.normal(size=(L, d)).astype(np.float32), P=None,
              A=rng.integers(-127, 128, size=(L, r, d)).astype(np.int8), B=np.ones((n, r), np.int8),
              scale_A=np.full(L, 0.01, np.float32), scale_B=np.full(L, 0.02, np.float32),
              cluster_offsets=np.array([0, 3000, 5000, 5000, n], np.int64), corpus=corpus, ids=None)
    q = rng.normal(size=(80, d)).astype(np.float32)          # (more than 64: the cluster-batched path)
    gix = B.Index(**ix)
    oix = O.OracleIndex(ix)
    for (k, w, m) in [(10, 3, 64), (5, 4, 200)]:
        o_ids, o_d, ost = O.search(oix, q, k, w, m, stages=True)
        g_ids, g_d, gst = gix.search_stages(q, k, w, m)
        np.testing.assert_array_equal(np.sort(gst["cand_rows"].astype(np.int64), axis=1), np.sort(ost["cand_rows"], axis=1))
        assert_topk_equal(g_ids, g_d, o_ids, o_d, "overflow")
        # a small batch finishes such queries inside its selection kernel
        s_ids, s_d, sst = gix.search_stages(q[:40], k, w, m)
        assert (sst["n_survivors"] == -1).any()
        np.testing.assert_array_equal(np.sort(sst["cand_rows"].astype(np.int64), axis=1), np.sort(ost["cand_rows"][:40], axis=1))
        np.testing.assert_array_equal(s_ids, g_ids[:40])
        np.testing.assert_array_equal(s_d, g_d[:40])
    # the count of queries finished by the per-query kernel, from synchronous, asynchronous and lane searches
    n_fb = int((gix.search_stages(q, 10, 3, 64)[2]["n_survivors"] == -1).sum())
    assert n_fb > 0
    gix.profile_enable(True)
    gix.search(q, 10, 3, 64)
    assert gix.profile_fallback_queries() == n_fb
    qd = torch.from_numpy(q).cuda()
    outs = [(torch.empty((80, 10), dtype=torch.int64, device="cuda"), torch.empty((80, 10), dtype=torch.float32, device="cuda")) for _ in range(3)]
    gix.search(qd, 10, 3, 64, out=outs[0], lane=1)
    gix.search(qd, 10, 3, 64, out=outs[1], lane=2)
    gix.search(qd, 10, 3, 64, out=outs[2], asynchronous=True)
    gix.lane_join(1); gix.lane_join(2)
    torch.cuda.synchronize()
    assert gix.profile_fallback_queries() == 4 * n_fb
    gix.profile_enable(False)
    gix.close()


def test_mixed_batch_some_queries_fall_back(B, small_indexes):
    """m close to the number of scored points and m / w beyond what the bound pass covers (no bound at all):
    both routes must agree with the oracle."""
    wl, ix, corpus, queries = small_indexes["ip_P"]
    a = ix.numpy()
    oix = O.OracleIndex(a)
    gix = B.Index.from_arrays(ix.to("cuda"))
    for (k, w, m) in [(10, 2, 70), (10, 1, 40), (10, 3, 1000), (10, wl.L, 2900), (3, 4, 31)]:
        o_ids, o_d, ost = O.search(oix, queries, k, w, m, stages=True)
        for reps in (1, 2):          # 40 queries: the query-major path of small batches; 80: the cluster-batched path
            g_ids, g_d, gst = gix.search_stages(np.tile(queries, (reps, 1)), k, w, m)
            np.testing.assert_array_equal(np.sort(gst["cand_rows"][:len(queries)].astype(np.int64), axis=1), np.sort(ost["cand_rows"], axis=1),
                                          err_msg=f"k={k} w={w} m={m} reps={reps}")
            assert_topk_equal(g_ids[:len(queries)], g_d[:len(queries)], o_ids, o_d, f"k={k} w={w} m={m} reps={reps}")
    gix.close()


@pytest.mark.parametrize("L,plateau", [(1500, 0), (4500, 0), (9000, 0), (9000, 3000), (16384, 0), (20000, 0)])
def test_many_clusters_routing_variants(B, L, plateau):
    """Cluster counts that take the other routing kernels (keys in 64 registers per lane; the row in the
    registers of a block; block-wide radix select), with duplicate centroids so that ties at the w-th place
    occur.  `plateau` > 0: that many identical centroids nearest to every query, more equal keys than the
    register kernel's candidate list holds, so it has to hand the row to the radix routine."""
    rng = np.random.default_rng(L + plateau)
    d, r, w = 32, 8, 40
    sizes = rng.integers(0, 7, size=L)
    n = int(sizes.sum())
    corpus = rng.normal(size=(n, d)).astype(np.float32)
    cent = rng.normal(size=(L, d)).astype(np.float32)
    cent[L // 2:L // 2 + 300] = cent[:300]                     # exact ties between cluster pairs
    if plateau:
        cent[1000:1000 + plateau] = 0.05 * rng.normal(size=d).astype(np.float32)
    off = np.zeros(L + 1, np.int64)
    np.cumsum(sizes, out=off[1:])
    ix = dict(metric=1, n=n, d=d, dp=d, r=r, L=L, centroids=cent, P=None,
              A=rng.integers(-127, 128, size=(L, r, d)).astype(np.int8), B=rng.integers(-127, 128, size=(n, r)).astype(np.int8),
              scale_A=rng.uniform(0.01, 0.1, L).astype(np.float32), scale_B=rng.uniform(0.01, 0.1, L).astype(np.float32),
              cluster_offsets=off, corpus=corpus, ids=None)
    q = rng.normal(size=(50, d)).astype(np.float32)
    if plateau:
        q *= 0.05                                              # short queries: the centroids near the origin win
    gix = B.Index(**ix)
    oix = O.OracleIndex(ix)
    o_ids, o_d, ost = O.search(oix, q, 10, w, 60, stages=True)
    if plateau:
        assert np.isin(ost["sel"], np.arange(1000, 1000 + plateau)).all()
    g_ids, g_d, gst = gix.search_stages(q, 10, w, 60)
    np.testing.assert_array_equal(gst["sel"], ost["sel"])
    np.testing.assert_array_equal(gst["z"], ost["z"])
    np.testing.assert_array_equal(np.sort(gst["cand_rows"].astype(np.int64), axis=1), np.sort(ost["cand_rows"], axis=1))
    assert_topk_equal(g_ids, g_d, o_ids, o_d, f"L={L} plateau={plateau}")
    gix.close()


def _sampled_full_size_parity(B, gix, a, queries, k, w, m, n_sample, tag, mixed=False):
    """One whole batch through lorann_search_stages and through the entry point the benchmark calls, then the oracle
    on a sample of the batch (it handles a query on its own, so any subset can be checked one by one): integer stages,
    per-pair best scores of the matrix-core kernel and candidate sets bit-exact, distances and ids to the usual bars."""
    g_ids, g_d, gst = gix.search_stages(queries, k, w, m)
    p_ids, p_d = gix.search(queries, k, w, m)
    np.testing.assert_array_equal(p_ids.cpu().numpy(), g_ids)
    np.testing.assert_array_equal(p_d.cpu().numpy(), g_d)
    nq = queries.shape[0]
    sample = np.sort(np.random.default_rng(7).choice(nq, size=min(n_sample, nq), replace=False))
    oix = O.OracleIndex(a)
    qh = queries.cpu().numpy()[sample]
    o_ids, o_d, ost = O.search(oix, qh, k, w, m, stages=True)
    np.testing.assert_array_equal(gst["qproj"][sample], ost["qproj"], err_msg=f"{tag}: projected queries")
    np.testing.assert_array_equal(gst["q8"][sample], ost["q8"], err_msg=f"{tag}: query codes")
    np.testing.assert_array_equal(gst["sel"][sample], ost["sel"], err_msg=f"{tag}: selected clusters")
    np.testing.assert_array_equal(gst["z"][sample], ost["z"], err_msg=f"{tag}: re-quantized vectors")
    np.testing.assert_array_equal(gst["sigma"][sample], ost["sigma"], err_msg=f"{tag}: pair scales")
    np.testing.assert_array_equal(gst["rho0"][sample], ost["rho0"], err_msg=f"{tag}: unquantized first components")
    np.testing.assert_array_equal(gst["pmax"][sample], ost["pair_best"], err_msg=f"{tag}: per-pair best scores (matrix-core kernel)")
    assert (np.abs(ost["rho0"]).max() > 0) == mixed
    np.testing.assert_array_equal(np.sort(gst["cand_rows"][sample].astype(np.int64), axis=1), np.sort(ost["cand_rows"], axis=1),
                                  err_msg=f"{tag}: candidate sets")
    assert_topk_equal(g_ids[sample], g_d[sample], o_ids, o_d, tag, abs_tol=rounding_abs_tol(qh, a["corpus"][:50000], a["metric"]),
                      exact=oracle_distance_of(a, qh))
    return gst


@pytest.mark.parametrize("workload,scheme,n_sample", [("embed-ip", "cluster", 192), ("embed-ip", "mixed", 192),
                                                      ("highdim-cos", "cluster", 96), ("lowdim-l2", "cluster", 96)])
def test_full_size_benchmark_configuration_sampled_parity(B, workload, scheme, n_sample):
    """(scheme: the configured step sizes per cluster, or the mixed-precision decomposition on column-wise step sizes.)
    The configured workloads at their full size - 1M x 768 inner product (the benchmark configuration: batch 10000,
    w=32, m=200), 1M x 1024 cosine (r=48, w=48, m=300: two k-steps on the matrix cores, rows of 4 KB in the re-rank),
    1M x 128 squared Euclidean without projection (r=24, w=64: the regime where a query's best estimates are spread over
    most of its clusters) - in the launch configuration bench.py times: device-resident inputs, one whole batch of
    10000 per call, hence the cluster-batched scoring, the per-query walk and the grouped re-rank with their
    full-size grids and work-item splits."""
    from paper_2410_18926_amd.synth import get_workload, make_dataset, build_index
    wl = get_workload(workload)
    dev = torch.device("cuda:0")
    corpus, queries = make_dataset(wl, dev)
    ix = build_index(corpus, wl, mixed_precision=(scheme == "mixed"))
    del corpus
    gix = B.Index.from_arrays(ix)
    a = ix.numpy()
    del ix
    torch.cuda.empty_cache()
    _sampled_full_size_parity(B, gix, a, queries, wl.k, wl.w, wl.m, n_sample, f"{workload} full size, {scheme}", mixed=(scheme == "mixed"))
    gix.close()


@pytest.mark.parametrize("metric", [0, 1, 2])
@pytest.mark.parametrize("nq", [1, 2, 17, 64])
def test_small_batches_take_the_query_major_path(B, nq, metric):
    """Batches of up to 64 queries skip the bucketing: one launch forms the first 8-bit product and re-quantizes it
    pair by pair in slot order, every pair is scored as a cluster of its own, a query whose survivor list overflows
    is finished in place, and the grouped re-rank takes the queries in their given order.  L = 16384
    clusters, w = 64, d' = 192, r = 32, m = 200 as in the 10M-point workload (150 000 points here), the three
    metrics; every stage against the oracle, and the same queries inside a larger batch (the cluster-batched
    path) give the same bits."""
    rng = np.random.default_rng(900 + 10 * metric + nq)
    ix = _random_index(rng, n=150_000, d=384, L=16384, r=32, metric=metric, dp=192)
    q = rng.normal(size=(nq, 384)).astype(np.float32)
    k, w, m = 10, 64, 200
    gix = B.Index(**ix)
    oix = O.OracleIndex(ix)
    o_ids, o_d, ost = O.search(oix, q, k, w, m, stages=True)
    yo = y_offsets(ost["sel"], ix["cluster_offsets"])
    g_ids, g_d, gst = gix.search_stages(q, k, w, m, y_off=yo)
    for key in ("qproj", "q8", "dx", "sel", "z", "sigma"):
        np.testing.assert_array_equal(gst[key], ost[key], err_msg=key)
    np.testing.assert_array_equal(gst["pmax"], ost["pair_best"], err_msg="per-pair best scores")
    y_ref = np.concatenate([O.pair_accumulators(ost["z"][s_ // w, s_ % w], ix["B"][ix["cluster_offsets"][c]:ix["cluster_offsets"][c + 1]])
                            for s_, c in enumerate(ost["sel"].reshape(-1))]) if yo[-1] else np.zeros(0, np.int32)
    np.testing.assert_array_equal(gst["y"], y_ref, err_msg="int32 accumulators")
    np.testing.assert_array_equal(np.sort(gst["cand_rows"].astype(np.int64), axis=1), np.sort(ost["cand_rows"], axis=1), err_msg="candidates")
    assert_topk_equal(g_ids, g_d, o_ids, o_d, f"nq={nq} metric={metric}", abs_tol=rounding_abs_tol(q, ix["corpus"], metric),
                      exact=oracle_distance_of(ix, q))
    big = np.concatenate([q, rng.normal(size=(70, 384)).astype(np.float32)])
    b_ids, b_d = gix.search(big, k, w, m)
    np.testing.assert_array_equal(b_ids[:nq], g_ids)
    np.testing.assert_array_equal(b_d[:nq], g_d)
    # device pointers, the asynchronous entry point and the one that allocates nothing
    qd = torch.from_numpy(q).cuda()
    for entry in ("async", "noalloc"):
        out = (torch.empty((nq, k), dtype=torch.int64, device="cuda"), torch.empty((nq, k), dtype=torch.float32, device="cuda"))
        if entry == "async":
            gix.search(qd, k, w, m, out=out, asynchronous=True)
        else:
            gix.search_noalloc(qd, k, w, m, out=out)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(out[0].cpu().numpy(), g_ids, err_msg=entry)
        np.testing.assert_array_equal(out[1].cpu().numpy(), g_d, err_msg=entry)
    gix.close()


@pytest.mark.parametrize("nq", [1024, 32768])
def test_many_clusters_full_launch_shapes_sampled_parity(B, nq):
    """The launch shapes of the 10M-point workload - L = 16384 clusters, w = 64, d' = 192, r = 32, m = 200, a batch of
    1024 (few pairs per cluster: the streaming shape of the scoring kernel, block-per-query cluster selection) and one
    whole chunk of 32768 queries (a 2 GB approximate-score matrix that is streamed past the caches, the dense scoring
    shape, 128 pairs per cluster on average) - on a corpus small enough for the host oracle (1M x 384, random factors
    and codes, clusters of 40..82 points), checked against the oracle on a sample of the batch."""
    from paper_2410_18926_amd.synth import get_workload, random_index
    import dataclasses
    wl = dataclasses.replace(get_workload("scale-ip"), n=1_000_000, nq=nq)
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(5150 + nq)
    corpus = torch.randn(wl.n, wl.d, generator=g, device=dev)
    corpus /= corpus.norm(dim=1, keepdim=True)
    queries = torch.randn(nq, wl.d, generator=g, device=dev)
    ix = random_index(corpus, wl)
    del corpus
    gix = B.Index.from_arrays(ix)
    a = ix.numpy()
    del ix
    torch.cuda.empty_cache()
    _sampled_full_size_parity(B, gix, a, queries, wl.k, wl.w, wl.m, 64, f"L=16384 launch shapes, nq={nq}")
    gix.close()


@pytest.mark.parametrize("metric,d,dp,L", [(1, 128, 128, 4096), (2, 320, 256, 4500), (0, 200, 128, 6000)])
def test_wide_launches_of_the_digest_screening_sampled_parity(B, metric, d, dp, L):
    """Launches large enough for the 512-query blocks of the screening passes (16384 queries) in the shapes the 10M-point
    workload does not cover: squared Euclidean (norms staged with the centroid tiles) and cosine, d' = 128 and 256 (the
    permuted tile layout), cluster counts that are no multiple of the tile - random factors and codes on 200 000 points,
    checked against the oracle on a sample of the batch."""
    from paper_2410_18926_amd.synth import get_workload, random_index
    import dataclasses
    nq = 16384
    wl = dataclasses.replace(get_workload("scale-ip"), n=200_000, d=d, dp=dp, L=L, metric=metric, nq=nq, w=32, m=100, r=16)
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(6100 + metric + dp)
    corpus = torch.randn(wl.n, wl.d, generator=g, device=dev)
    if metric == 2:
        corpus /= corpus.norm(dim=1, keepdim=True)
    queries = torch.randn(nq, wl.d, generator=g, device=dev)
    ix = random_index(corpus, wl)
    del corpus
    gix = B.Index.from_arrays(ix)
    a = ix.numpy()
    del ix
    torch.cuda.empty_cache()
    _sampled_full_size_parity(B, gix, a, queries, wl.k, wl.w, wl.m, 48, f"wide digest launch metric={metric} d'={dp} L={L}")
    gix.set_screen_mode(B.SCREEN_MATRIX)
    m_ids, m_d, mst = gix.search_stages(queries[:4096], wl.k, wl.w, wl.m)
    gix.set_screen_mode(B.SCREEN_AUTO)
    d_ids, d_d, dst = gix.search_stages(queries, wl.k, wl.w, wl.m)
    np.testing.assert_array_equal(dst["sel"][:4096], mst["sel"])
    gix.close()


@pytest.mark.parametrize("L,w,metric,case", [
    (700, 32, 0, "near_ties"), (700, 32, 1, "near_ties"), (700, 32, 2, "plateau"), (512, 100, 0, "plain"),
    (512, 100, 1, "near_ties"), (900, 40, 0, "outlier"), (900, 40, 1, "outlier"), (64, 64, 0, "plain"),
    (3000, 48, 0, "near_ties"), (3000, 48, 1, "outlier"), (12000, 64, 0, "near_ties"), (12000, 200, 2, "plain"),
])
def test_routing_by_screening_adversarial(B, L, w, metric, case):
    """Routing finds the w nearest centroids from bfloat16 scores plus an error bound and evaluates only a short
    list exactly.  These inputs stress the list: hundreds of centroids within 1e-6 of each other around the
    w-th place (near_ties), several hundred identical ones (plateau: the list overflows and every cluster is
    evaluated exactly), one centroid of huge norm (outlier: the bound becomes useless), w above the lane count.
    The selected clusters must equal the oracle's, in order, whatever route is taken."""
    rng = np.random.default_rng(1000 * L + w + metric)
    d, r = 32, 8
    sizes = rng.integers(1, 5, size=L)
    n = int(sizes.sum())
    corpus = rng.normal(size=(n, d)).astype(np.float32)
    cent = rng.normal(size=(L, d)).astype(np.float32)
    cent /= np.linalg.norm(cent, axis=1, keepdims=True)
    q = rng.normal(size=(40, d)).astype(np.float32)
    q /= np.linalg.norm(q, axis=1, keepdims=True)
    if case == "near_ties":
        # 300 centroids that differ from one direction by ~1e-6: their scores crowd around the w-th place
        base = q[0] / np.linalg.norm(q[0])
        idx = rng.choice(L, size=min(300, L // 2), replace=False)
        cent[idx] = (base[None, :] * (1.0 + 1e-6 * rng.normal(size=(idx.size, 1))) + 1e-6 * rng.normal(size=(idx.size, d))).astype(np.float32)
        q[1:20] = (base[None, :] + 0.05 * rng.normal(size=(19, d))).astype(np.float32)
    elif case == "plateau":
        idx = rng.choice(L, size=400, replace=False)
        cent[idx] = q[0]
        q[1:20] = (q[0][None, :] + 0.01 * rng.normal(size=(19, d))).astype(np.float32)
    elif case == "outlier":
        cent[L // 3] *= 3.0e4
        cent[L // 3 + 1] *= -2.0e4
    if metric == 2:
        corpus /= np.linalg.norm(corpus, axis=1, keepdims=True)
    off = np.zeros(L + 1, np.int64)
    np.cumsum(sizes, out=off[1:])
    ix = dict(metric=metric, n=n, d=d, dp=d, r=r, L=L, centroids=cent, P=None,
              A=rng.integers(-127, 128, size=(L, r, d)).astype(np.int8), B=rng.integers(-127, 128, size=(n, r)).astype(np.int8),
              scale_A=rng.uniform(0.01, 0.1, L).astype(np.float32), scale_B=rng.uniform(0.01, 0.1, L).astype(np.float32),
              cluster_offsets=off, corpus=corpus, ids=None)
    gix = B.Index(**ix)
    oix = O.OracleIndex(ix)
    m = 50
    o_ids, o_d, ost = O.search(oix, q, 10, w, m, stages=True)
    g_ids, g_d, gst = gix.search_stages(q, 10, w, m)
    np.testing.assert_array_equal(gst["sel"], ost["sel"], err_msg=f"selected clusters ({case})")
    np.testing.assert_array_equal(gst["z"], ost["z"])
    assert_topk_equal(g_ids, g_d, o_ids, o_d, f"L={L} w={w} metric={metric} {case}")
    # the plain route (all L dissimilarities in double) agrees as well
    gix.set_exact_selection(True)
    e_ids, e_d, est = gix.search_stages(q, 10, w, m)
    np.testing.assert_array_equal(est["sel"], ost["sel"], err_msg=f"selected clusters, plain route ({case})")
    gix.close()


@pytest.mark.parametrize("L,w,metric,dp,nq,case", [
    (2048, 32, 0, 128, 40, "plain"), (2500, 64, 1, 128, 300, "near_ties"), (2500, 48, 2, 192, 70, "plateau"),
    (12000, 64, 0, 192, 300, "near_ties"), (12000, 128, 1, 192, 40, "plain"), (16384, 64, 0, 192, 600, "plain"),
    (5000, 40, 0, 128, 40, "outlier"), (5000, 40, 1, 192, 40, "outlier"), (4097, 100, 2, 128, 129, "near_ties"),
    (3000, 48, 0, 256, 300, "near_ties"), (9000, 64, 1, 256, 70, "plain"), (2049, 32, 2, 256, 600, "plateau"),
    (1024, 128, 0, 128, 513, "plain"), (1100, 16, 1, 192, 512, "plain"), (1500, 1, 2, 128, 65, "plain"),
])
def test_routing_by_screening_from_digests(B, L, w, metric, dp, nq, case):
    """The screening that never writes the nq x L matrix of approximate values (two passes of the bf16 product: minima
    of 256 subsets of the clusters, then lists of the values below a per-query threshold), forced for batches far
    smaller than those that take it by themselves.  Cluster counts that are no multiple of the 64-cluster tile or of
    the 16 runs, batches that end inside a wavefront's 64 queries, and the inputs that stress the lists: hundreds of
    centroids within 1e-6 of each other (near_ties), 400 identical ones (plateau: a lane's list or the block's list
    overflows, every cluster is evaluated exactly), centroids of huge norm (outlier: the bound is useless, everything
    is listed).  The selected clusters must equal the oracle's, in order, and those of the matrix route."""
    rng = np.random.default_rng(77 * L + w + metric + nq)
    d, r = (dp, 8) if metric != 0 else (dp + 40, 8)          # inner product: with a projection
    sizes = rng.integers(1, 4, size=L)
    n = int(sizes.sum())
    corpus = rng.normal(size=(n, d)).astype(np.float32)
    cent = rng.normal(size=(L, dp)).astype(np.float32)
    cent /= np.linalg.norm(cent, axis=1, keepdims=True)
    P = None if dp == d else np.linalg.qr(rng.normal(size=(d, d)))[0][:, :dp].astype(np.float32)
    q = rng.normal(size=(nq, d)).astype(np.float32)
    q /= np.linalg.norm(q, axis=1, keepdims=True)
    qp0 = q[0] if P is None else (q[0].astype(np.float64) @ P.astype(np.float64)).astype(np.float32)
    base = qp0 / np.linalg.norm(qp0)
    if case == "near_ties":
        idx = rng.choice(L, size=300, replace=False)
        cent[idx] = (base[None, :] * (1.0 + 1e-6 * rng.normal(size=(idx.size, 1))) + 1e-6 * rng.normal(size=(idx.size, dp))).astype(np.float32)
        q[1:20] = q[0][None, :] + 0.05 * rng.normal(size=(19, d)).astype(np.float32)
    elif case == "plateau":
        idx = rng.choice(L, size=400, replace=False)
        cent[idx] = base
        q[1:20] = q[0][None, :] + 0.01 * rng.normal(size=(19, d)).astype(np.float32)
    elif case == "outlier":
        cent[L // 3] *= 3.0e4
        cent[L // 3 + 1] *= -2.0e4
    if metric == 2:
        corpus /= np.linalg.norm(corpus, axis=1, keepdims=True)
    off = np.zeros(L + 1, np.int64)
    np.cumsum(sizes, out=off[1:])
    ix = dict(metric=metric, n=n, d=d, dp=dp, r=r, L=L, centroids=cent, P=P,
              A=rng.integers(-127, 128, size=(L, r, dp)).astype(np.int8), B=rng.integers(-127, 128, size=(n, r)).astype(np.int8),
              scale_A=rng.uniform(0.01, 0.1, L).astype(np.float32), scale_B=rng.uniform(0.01, 0.1, L).astype(np.float32),
              cluster_offsets=off, corpus=corpus, ids=None)
    gix = B.Index(**ix)
    oix = O.OracleIndex(ix)
    m = 50
    o_ids, o_d, ost = O.search(oix, q, 10, w, m, stages=True)
    gix.set_screen_mode(B.SCREEN_DIGEST)
    g_ids, g_d, gst = gix.search_stages(q, 10, w, m)
    np.testing.assert_array_equal(gst["sel"], ost["sel"], err_msg=f"selected clusters ({case})")
    np.testing.assert_array_equal(gst["q8"], ost["q8"])
    np.testing.assert_array_equal(gst["z"], ost["z"])
    assert_topk_equal(g_ids, g_d, o_ids, o_d, f"digests: L={L} w={w} metric={metric} {case}")
    gix.set_screen_mode(B.SCREEN_MATRIX)
    m_ids, m_d, mst = gix.search_stages(q, 10, w, m)
    np.testing.assert_array_equal(mst["sel"], gst["sel"])
    np.testing.assert_array_equal(m_ids, g_ids)
    np.testing.assert_array_equal(m_d, g_d)
    with pytest.raises(B.LorannError):
        gix.set_screen_mode(7)
    gix.close()


def _random_index(rng, n, d, L, r, metric, dp=None, with_ids=True):
    dp = dp or d
    cuts = np.sort(rng.choice(np.arange(1, n), size=L - 1, replace=False))
    off = np.concatenate([[0], cuts, [n]]).astype(np.int64)
    corpus = rng.normal(size=(n, d)).astype(np.float32)
    if metric == 2:
        corpus /= np.linalg.norm(corpus, axis=1, keepdims=True)
    P = None if dp == d else np.linalg.qr(rng.normal(size=(d, d)))[0][:, :dp].astype(np.float32)
    return dict(metric=metric, n=n, d=d, dp=dp, r=r, L=L, centroids=rng.normal(size=(L, dp)).astype(np.float32), P=P,
                A=rng.integers(-127, 128, size=(L, r, dp)).astype(np.int8), B=rng.integers(-127, 128, size=(n, r)).astype(np.int8),
                scale_A=rng.uniform(0.01, 0.1, L).astype(np.float32), scale_B=rng.uniform(0.01, 0.1, L).astype(np.float32),
                cluster_offsets=off, corpus=corpus, ids=rng.permutation(n).astype(np.int64) if with_ids else None)


@pytest.mark.parametrize("metric", [0, 1, 2])
def test_parameter_extremes(B, metric):
    """Parameters at and across the internal switch points: k at 64 / 65 (wavefront vs block top-k), m at 256 / 300 /
    512 / 513 / 1025 / 4096 (top-k register budget, grouped vs one-query re-rank, the two capacities of the
    per-query walk), w = 256 of 300 clusters."""
    rng = np.random.default_rng(70 + metric)
    ix = _random_index(rng, n=6000, d=48, L=300, r=16, metric=metric, dp=32)
    q = rng.normal(size=(37, 48)).astype(np.float32)
    gix = B.Index(**ix)
    oix = O.OracleIndex(ix)
    for (k, w, m) in [(64, 20, 256), (65, 20, 300), (100, 30, 512), (10, 30, 513), (200, 40, 1025), (10, 256, 4096), (1, 256, 200)]:
        o_ids, o_d, ost = O.search(oix, q, k, w, m, stages=True)
        g_ids, g_d, gst = gix.search_stages(q, k, w, m)
        np.testing.assert_array_equal(gst["sel"], ost["sel"], err_msg=f"k={k} w={w} m={m}")
        np.testing.assert_array_equal(np.sort(gst["cand_rows"].astype(np.int64), axis=1), np.sort(ost["cand_rows"], axis=1),
                                      err_msg=f"candidate sets k={k} w={w} m={m}")
        assert_topk_equal(g_ids, g_d, o_ids, o_d, f"metric={metric} k={k} w={w} m={m}")
    gix.close()


@pytest.mark.parametrize("d", [1028, 1100, 2000])
def test_long_rows(B, d):
    """Rows longer than the register-resident re-rank handles (d > 1024: streamed rows) and longer than a group of
    queries fits in LDS (d = 2000: one query per block)."""
    rng = np.random.default_rng(d)
    ix = _random_index(rng, n=1500, d=d, L=12, r=8, metric=1, dp=64)
    q = rng.normal(size=(21, d)).astype(np.float32)
    gix = B.Index(**ix)
    oix = O.OracleIndex(ix)
    o_ids, o_d = O.search(oix, q, 10, 5, 120)
    g_ids, g_d = gix.search(q, 10, 5, 120)
    assert_topk_equal(g_ids, g_d, o_ids, o_d, f"d={d}")
    gix.close()


def test_batch_larger_than_one_launch(B):
    """A batch of 70 000 queries runs as three launches of at most 32 768; every query must come out as if alone."""
    rng = np.random.default_rng(33)
    ix = _random_index(rng, n=3000, d=16, L=40, r=8, metric=0, with_ids=False)
    q = rng.normal(size=(70000, 16)).astype(np.float32)
    gix = B.Index(**ix)
    oix = O.OracleIndex(ix)
    g_ids, g_d = gix.search(torch.from_numpy(q).cuda(), 5, 4, 30)
    g_ids, g_d = g_ids.cpu().numpy(), g_d.cpu().numpy()
    pick = np.concatenate([np.arange(0, 64), np.arange(32768 - 32, 32768 + 32), np.arange(65536 - 32, 65536 + 32), np.arange(70000 - 64, 70000)])
    o_ids, o_d = O.search(oix, q[pick], 5, 4, 30)
    assert_topk_equal(g_ids[pick], g_d[pick], o_ids, o_d, "chunked batch")
    # and the whole batch equals the same queries searched in small pieces
    h_ids, h_d = gix.search(torch.from_numpy(q[40000:41000]).cuda(), 5, 4, 30)
    np.testing.assert_array_equal(h_ids.cpu().numpy(), g_ids[40000:41000])
    np.testing.assert_array_equal(h_d.cpu().numpy(), g_d[40000:41000])
    gix.close()


def test_asynchronous_searches_match_synchronous_ones(B, small_indexes):
    """lorann_search_async enqueues and returns: several calls in a row on different buffers, synchronised once,
    must give what the synchronous entry point gives; host pointers are refused."""
    wl, ix, corpus, queries = small_indexes["ip_P"]
    gix = B.Index.from_arrays(ix.to("cuda"))
    gix.use_torch_stream()
    k, w, m = wl.k, wl.w, wl.m
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(12)
    sets = [torch.from_numpy(queries[rng.choice(queries.shape[0], size=n, replace=True)]).to(dev) for n in (33, 200, 7, 129)]
    outs = [(torch.empty((q.shape[0], k), dtype=torch.int64, device=dev), torch.empty((q.shape[0], k), dtype=torch.float32, device=dev)) for q in sets]
    gix.profile_enable(True)
    for q, o in zip(sets, outs):
        gix.search(q, k, w, m, out=o, asynchronous=True)
    torch.cuda.synchronize()
    prof = gix.profile_get()
    assert prof["rerank"][1] == len(sets)                 # the pending events of all four calls were collected
    gix.profile_enable(False)
    for q, o in zip(sets, outs):
        s_ids, s_d = gix.search(q, k, w, m)
        np.testing.assert_array_equal(o[0].cpu().numpy(), s_ids.cpu().numpy())
        np.testing.assert_array_equal(o[1].cpu().numpy(), s_d.cpu().numpy())
    with pytest.raises(B.LorannError):
        gix.search(queries[:4], k, w, m, asynchronous=True)
    gix.close()


def test_half_precision_rerank_small_workloads(B, small_indexes):
    """Re-rank over the binary16 copy of the corpus (Sec. 4.3): the library's rounding and float arithmetic against
    the oracle's plain re-rank over numpy-rounded rows; candidates are those of the float mode; switching back
    restores the float results."""
    for name, (wl, ix, corpus, queries) in small_indexes.items():
        a = ix.numpy()
        o_ids, o_d, ost = O.search(O.OracleIndex(O.with_half_precision_corpus(a)), queries, wl.k, wl.w, wl.m, stages=True)
        gix = B.Index.from_arrays(ix.to("cuda"))
        f_ids, f_d = gix.search(queries, wl.k, wl.w, wl.m)
        gix.set_rerank(B.RERANK_F16)
        g_ids, g_d, gst = gix.search_stages(queries, wl.k, wl.w, wl.m)
        np.testing.assert_array_equal(np.sort(gst["cand_rows"].astype(np.int64), axis=1), np.sort(ost["cand_rows"], axis=1), err_msg=name)
        assert_topk_equal(g_ids, g_d, o_ids, o_d, f"{name} half-precision rows")
        gix.set_exact_selection(True)                       # the one-query-per-block re-rank reads the same copy
        e_ids, e_d = gix.search(queries, wl.k, wl.w, wl.m)
        gix.set_exact_selection(False)
        np.testing.assert_array_equal(e_ids, g_ids)
        np.testing.assert_array_equal(e_d, g_d)
        gix.set_rerank(B.RERANK_F32)
        b_ids, b_d = gix.search(queries, wl.k, wl.w, wl.m)
        np.testing.assert_array_equal(b_ids, f_ids)
        np.testing.assert_array_equal(b_d, f_d)
        gix.close()


@pytest.mark.parametrize("d,metric", [(768, 0), (1024, 1), (200, 2), (50, 1), (1100, 0), (2000, 1)])
def test_half_precision_rerank_row_lengths(B, d, metric):
    """Every row-length path of the gather (one to four register slices, rows not a multiple of four elements,
    streamed rows, one query per block), values spread over binary16's normal and subnormal ranges."""
    rng = np.random.default_rng(1000 + d)
    ix = _random_index(rng, n=2500, d=d, L=16, r=8, metric=metric, dp=64 if d >= 64 else 32)
    if metric != 2:
        ix["corpus"] = (ix["corpus"] * np.exp(rng.normal(size=(2500, 1)) * 2).astype(np.float32)).astype(np.float32)
        ix["corpus"][::97, ::5] *= np.float32(1e-6)        # binary16 subnormals and zeros
    q = rng.normal(size=(45, d)).astype(np.float32)
    gix = B.Index(**ix)
    gix.set_rerank(B.RERANK_F16)
    o_ids, o_d = O.search(O.OracleIndex(O.with_half_precision_corpus(ix)), q, 10, 6, 150)
    g_ids, g_d = gix.search(q, 10, 6, 150)
    assert_topk_equal(g_ids, g_d, o_ids, o_d, f"d={d} metric={metric} half-precision rows")
    gix.close()


@pytest.mark.parametrize("d,metric,nq,m,half", [(64, 1, 1, 100, False), (300, 0, 5, 60, False), (768, 2, 8, 200, False), (1024, 0, 3, 300, True),
                                               (1024, 1, 8, 512, False), (96, 2, 2, 40, True), (1028, 0, 4, 100, False), (64, 0, 2, 600, False)])
def test_a_handful_of_queries_rerank_in_one_launch(B, d, metric, nq, m, half):
    """Up to eight queries: the re-rank computes distances and orders the results in ONE launch (blocks per query,
    the last one to finish orders).  One to four register slices per row, float and half-precision rows, caller ids,
    fewer than m candidates, a row length and a candidate count (m = 600) that take the general path instead; against
    the oracle, and the same
    queries inside a batch of 100 (grouped gather + separate top-k) must give the same bits."""
    rng = np.random.default_rng(5000 + d + metric + nq)
    ix = _random_index(rng, n=1500, d=d, L=12, r=8, metric=metric, dp=64 if d >= 64 else 32)
    if half and metric != 2:
        ix["corpus"] = (ix["corpus"] * np.float32(0.25)).astype(np.float32)
    big = rng.normal(size=(100, d)).astype(np.float32)
    q = big[:nq].copy()
    w, k = (2 if m >= 300 else 5), 10         # (two clusters of about 125 points: fewer than m candidates)
    gix = B.Index(**ix)
    if half:
        gix.set_rerank(B.RERANK_F16)
    for rep in range(2):                      # twice: the tickets of the first call must not linger
        s_ids, s_d, sst = gix.search_stages(q, k, w, m)
        b_ids, b_d = gix.search(big, k, w, m)
        np.testing.assert_array_equal(s_ids, b_ids[:nq])
        np.testing.assert_array_equal(s_d.view(np.uint32), b_d[:nq].view(np.uint32))
    if m >= 300:
        assert (sst["cand_rows"] < 0).any(), "the case is meant to have queries with fewer than m candidates"
    o_ids, o_d = O.search(O.OracleIndex(O.with_half_precision_corpus(ix) if half else ix), q, k, w, m)
    assert_topk_equal(s_ids, s_d, o_ids, o_d, f"handful d={d} metric={metric} nq={nq} half={half}")
    gix.close()


def test_rows_requested_by_the_grouped_rerank_are_counted(B):
    """lorann_profile_gather_rows (the numerator of the benchmark's roofline): the rows the last grouped re-rank fetched
    lie between the distinct candidate rows of the batch (every row at least once) and the candidates themselves (no
    sharing at all); with one query per group (a batch of 40 takes groups of one) it is exactly the candidates."""
    rng = np.random.default_rng(321)
    ix = _random_index(rng, n=4000, d=64, L=10, r=8, metric=0, dp=32)
    gix = B.Index(**ix)
    for nq in (200, 40):
        q = rng.normal(size=(nq, 64)).astype(np.float32)
        q[1::2] = q[0::2] + np.float32(0.01) * rng.normal(size=(nq // 2, 64)).astype(np.float32)     # neighbours share rows
        ids, d, st = gix.search_stages(q, 10, 4, 120)
        gix.search(q, 10, 4, 120)
        rows = gix.profile_gather_rows()
        cand = st["cand_rows"]
        valid = int((cand >= 0).sum())
        distinct = int(np.unique(cand[cand >= 0]).size)
        if nq == 40:
            assert rows == valid
        else:
            assert distinct <= rows < valid, (distinct, rows, valid)
    gix.close()


def test_half_precision_rerank_refuses_values_out_of_range(B):
    rng = np.random.default_rng(77)
    ix = _random_index(rng, n=600, d=32, L=6, r=8, metric=0)
    q = rng.normal(size=(9, 32)).astype(np.float32)
    for bad in (7.0e4, -1.0e9, np.inf, np.nan):
        broken = dict(ix)
        broken["corpus"] = ix["corpus"].copy()
        broken["corpus"][311, 7] = bad
        gix = B.Index(**broken)
        with pytest.raises(B.LorannError) as ei:
            gix.set_rerank(B.RERANK_F16)
        assert ei.value.code == B.LORANN_E_UNSUPPORTED
        if np.isfinite(bad):                                # the mode is unchanged: float rows are still what is read
            o_ids, o_d = O.search(O.OracleIndex(broken), q, 5, 3, 40)
            g_ids, g_d = gix.search(q, 5, 3, 40)
            assert_topk_equal(g_ids, g_d, o_ids, o_d, f"after refusing {bad}")
        gix.close()
    edge = dict(ix)
    edge["corpus"] = ix["corpus"].copy()
    edge["corpus"][5, 5] = 65504.0                          # the largest binary16 value is fine
    gix = B.Index(**edge)
    gix.set_rerank(B.RERANK_F16)
    with pytest.raises(B.LorannError):
        gix.set_rerank(7)
    gix.close()


def test_search_without_rerank_small_workloads(B, small_indexes):
    """No re-ranking step (Sec. 7.1 memory usage, App. D.3): ids and -score bit-identical to the oracle's, from the
    batched selection and from the per-query kernel, with m ignored."""
    for name, (wl, ix, corpus, queries) in small_indexes.items():
        a = ix.numpy()
        oix = O.OracleIndex(a)
        gix = B.Index.from_arrays(ix.to("cuda"))
        gix.set_rerank(B.RERANK_NONE)
        for k in (1, wl.k, 64, 70):
            o_ids, o_d = O.search_no_rerank(oix, queries, k, wl.w)
            g_ids, g_d = gix.search(queries, k, wl.w, max(k, wl.m))
            np.testing.assert_array_equal(g_ids, o_ids, err_msg=f"{name} k={k}")
            np.testing.assert_array_equal(g_d, o_d, err_msg=f"{name} k={k}")
            gix.set_exact_selection(True)
            e_ids, e_d = gix.search(queries, k, wl.w, max(k, wl.m))
            gix.set_exact_selection(False)
            np.testing.assert_array_equal(e_ids, o_ids, err_msg=f"{name} k={k} per-query kernel")
            np.testing.assert_array_equal(e_d, o_d, err_msg=f"{name} k={k} per-query kernel")
        gix.close()


def test_search_without_rerank_ties_and_short_lists(B):
    """Many equal scores (tiny codes): boundary ties go to the lower row, reported ties to the lower id; fewer scored
    points than k pads with -1 / +inf."""
    rng = np.random.default_rng(8)
    ix = _random_index(rng, n=900, d=32, L=30, r=8, metric=0)
    ix["B"] = rng.integers(-1, 2, size=ix["B"].shape).astype(np.int8)
    ix["cluster_offsets"] = np.concatenate([[0, 0, 3, 3, 5], np.linspace(40, 900, 26).astype(np.int64)])
    q = rng.normal(size=(60, 32)).astype(np.float32)
    gix = B.Index(**ix)
    gix.set_rerank(B.RERANK_NONE)
    oix = O.OracleIndex(ix)
    for k, w in [(10, 5), (100, 2), (40, 30), (300, 1)]:
        o_ids, o_d = O.search_no_rerank(oix, q, k, w)
        g_ids, g_d = gix.search(q, k, w, k)
        np.testing.assert_array_equal(g_ids, o_ids, err_msg=f"k={k} w={w}")
        np.testing.assert_array_equal(g_d, o_d, err_msg=f"k={k} w={w}")
    gix.close()


def test_column_scales_small_workloads_stagewise(B, small_indexes_columns):
    """Column-wise quantization (Sec. 3.3 as printed: one step size per column of A_c and of B_c): every stage
    bit-exact against the oracle - float re-quantization of the first product included - on the four small
    configurations, through the batched path and the per-query kernel."""
    for name, (wl, ix, corpus, queries) in small_indexes_columns.items():
        _stagewise(B, wl, ix, queries)


@pytest.mark.parametrize("r,dp,metric,dense", [(8, 16, 0, False), (24, 48, 1, False), (32, 256, 0, True), (48, 64, 2, False),
                                               (64, 128, 1, True), (16, 1024, 0, False)])
def test_column_scales_rank_dimension_metric_variants(B, r, dp, metric, dense):
    """Random factors with widely spread step sizes (four decades across columns and across points), ranks that pad
    on the matrix cores, both regimes of the pair-maxima kernel (dense: many pairs per cluster; else few), zero step
    sizes (a dead column, a dead point).  Candidates bit-exact; also the search without re-ranking."""
    rng = np.random.default_rng(500 + r + metric)
    n, L, nq = (4000, 6, 300) if dense else (3000, 40, 45)
    ix = _random_index(rng, n=n, d=dp, L=L, r=r, metric=metric)
    ix["scale_A_columns"] = (10.0 ** rng.uniform(-4, 0, size=(L, r))).astype(np.float32)
    ix["scale_B_points"] = (10.0 ** rng.uniform(-4, 0, size=n)).astype(np.float32)
    ix["scale_A_columns"][1, 3] = 0.0
    ix["scale_B_points"][17] = 0.0
    ix["scale_A_columns"][2, :] = 0.0                         # a cluster whose intermediate vector is all zero
    q = rng.normal(size=(nq, dp)).astype(np.float32)
    w, m, k = min(L, 5), 60, 10
    oix = O.OracleIndex(ix)
    o_ids, o_d, ost = O.search(oix, q, k, w, m, stages=True)
    gix = B.Index(**ix)
    g_ids, g_d, gst = gix.search_stages(q, k, w, m)
    np.testing.assert_array_equal(gst["z"], ost["z"], err_msg="re-quantized vectors")
    np.testing.assert_array_equal(gst["sigma"], ost["sigma"], err_msg="pair step sizes")
    np.testing.assert_array_equal(gst["pmax"], ost["pair_best"], err_msg="per-pair best scores (matrix-core kernel)")
    np.testing.assert_array_equal(np.sort(gst["cand_rows"].astype(np.int64), axis=1), np.sort(ost["cand_rows"], axis=1), err_msg="candidates")
    assert_topk_equal(g_ids, g_d, o_ids, o_d, "column scales", abs_tol=rounding_abs_tol(q, ix["corpus"], metric), exact=oracle_distance_of(ix, q))
    gix.set_exact_selection(True)
    e_ids, e_d, est = gix.search_stages(q, k, w, m)
    gix.set_exact_selection(False)
    np.testing.assert_array_equal(np.sort(est["cand_rows"].astype(np.int64), axis=1), np.sort(ost["cand_rows"], axis=1), err_msg="candidates (per-query kernel)")
    gix.set_rerank(B.RERANK_NONE)
    n_ids, n_d = gix.search(q, k, w, k)
    r_ids, r_d = O.search_no_rerank(oix, q, k, w)
    np.testing.assert_array_equal(n_ids, r_ids)
    np.testing.assert_array_equal(n_d, r_d)
    gix.close()


def test_column_scales_can_be_set_and_removed(B, small_indexes, small_indexes_columns):
    """lorann_set_column_scales on a loaded index, back to per-cluster step sizes with NULLs, and its refusals."""
    wl, ixc, corpus, queries = small_indexes_columns["ip_P"]
    a = ixc.numpy()
    plain = {k: v for k, v in a.items() if k not in ("scale_A_columns", "scale_B_points")}
    gix = B.Index(**plain)
    p_ids, p_d = gix.search(queries, wl.k, wl.w, wl.m)                      # the codes read with the per-cluster step sizes
    o_ids, o_d = O.search(O.OracleIndex(plain), queries, wl.k, wl.w, wl.m)
    assert_topk_equal(p_ids, p_d, o_ids, o_d, "per-cluster reading")
    gix.set_column_scales(a["scale_A_columns"], torch.from_numpy(a["scale_B_points"]).cuda())   # host and device pointers
    c_ids, c_d, cst = gix.search_stages(queries, wl.k, wl.w, wl.m)
    oc_ids, oc_d, ost = O.search(O.OracleIndex(a), queries, wl.k, wl.w, wl.m, stages=True)
    np.testing.assert_array_equal(cst["z"], ost["z"])
    assert_topk_equal(c_ids, c_d, oc_ids, oc_d, "column-wise reading")
    for bad_a, bad_b in [(a["scale_A_columns"], None), (None, a["scale_B_points"]),
                         (-a["scale_A_columns"] - 1, a["scale_B_points"]), (a["scale_A_columns"], a["scale_B_points"] * np.float32(np.nan))]:
        with pytest.raises(B.LorannError) as ei:
            gix.set_column_scales(bad_a, bad_b)
        assert ei.value.code == B.LORANN_E_INVAL
    k_ids, k_d = gix.search(queries, wl.k, wl.w, wl.m)                      # a refused call changes nothing
    np.testing.assert_array_equal(k_ids, c_ids)
    gix.set_column_scales(None, None)
    b_ids, b_d = gix.search(queries, wl.k, wl.w, wl.m)
    np.testing.assert_array_equal(b_ids, p_ids)
    np.testing.assert_array_equal(b_d, p_d)
    gix.close()


def test_mixed_precision_small_workloads_stagewise(B, small_indexes_mixed):
    """Mixed-precision decomposition (Sec. 4.2: the first component of the projected query and the first rows of A_c
    and B_c stay in float): every stage bit-exact against the oracle - the codes that skip the first component, the
    float first component of every pair's intermediate vector, the candidates - on the four small configurations,
    through the batched path and the per-query kernel."""
    for name, (wl, ix, corpus, queries) in small_indexes_mixed.items():
        assert ix.first_row_A is not None and float(ix.first_row_B.abs().max()) > 0
        _stagewise(B, wl, ix, queries)


@pytest.mark.parametrize("r,dp,metric,dense", [(8, 16, 0, False), (24, 48, 1, False), (32, 256, 0, True), (48, 64, 2, False),
                                               (64, 128, 1, True), (16, 1024, 0, False), (8, 512, 2, True)])
def test_mixed_precision_rank_dimension_metric_variants(B, r, dp, metric, dense):
    """Random factors, float first rows whose size ranges from negligible to dominant against the quantized rest,
    non-zero codes in the positions that must not be read, ranks that pad on the matrix cores, both regimes of the pair-maxima kernel.  Stages and candidates bit-exact; also the search
    without re-ranking."""
    rng = np.random.default_rng(900 + r + metric)
    n, L, nq = (4000, 6, 300) if dense else (3000, 40, 45)
    ix = _random_index(rng, n=n, d=dp, L=L, r=r, metric=metric)
    ix["scale_A_columns"] = (10.0 ** rng.uniform(-3, 0, size=(L, r))).astype(np.float32)
    ix["scale_B_points"] = (10.0 ** rng.uniform(-3, 0, size=n)).astype(np.float32)
    ix["first_row_A"] = (rng.normal(size=(L, r)) * 10.0 ** rng.uniform(-2, 2, size=(L, 1))).astype(np.float32)
    ix["first_row_B"] = (rng.normal(size=n) * 10.0 ** rng.uniform(-2, 2, size=n)).astype(np.float32)
    ix["first_row_A"][1, :] = 0.0
    ix["first_row_B"][5] = 0.0
    q = rng.normal(size=(nq, dp)).astype(np.float32)
    q[:, 0] *= 30.0                                              # the component that would otherwise set the step size
    q[3, 1:] = 0.0                                               # nothing but the first component
    q[4, 0] = 0.0
    w, m, k = min(L, 5), 60, 10
    oix = O.OracleIndex(ix)
    o_ids, o_d, ost = O.search(oix, q, k, w, m, stages=True)
    assert not ost["q8"][:, 0].any() and not ost["z"][:, :, 0].any()
    gix = B.Index(**ix)
    g_ids, g_d, gst = gix.search_stages(q, k, w, m)
    np.testing.assert_array_equal(gst["q8"], ost["q8"], err_msg="query codes")
    np.testing.assert_array_equal(gst["dx"], ost["dx"], err_msg="query step sizes")
    np.testing.assert_array_equal(gst["rho0"], ost["rho0"], err_msg="unquantized first components")
    np.testing.assert_array_equal(gst["z"], ost["z"], err_msg="re-quantized vectors")
    np.testing.assert_array_equal(gst["sigma"], ost["sigma"], err_msg="pair step sizes")
    np.testing.assert_array_equal(gst["pmax"], ost["pair_best"], err_msg="per-pair best scores (matrix-core kernel)")
    np.testing.assert_array_equal(np.sort(gst["cand_rows"].astype(np.int64), axis=1), np.sort(ost["cand_rows"], axis=1), err_msg="candidates")
    assert_topk_equal(g_ids, g_d, o_ids, o_d, "mixed precision", abs_tol=rounding_abs_tol(q, ix["corpus"], metric), exact=oracle_distance_of(ix, q))
    gix.set_exact_selection(True)
    e_ids, e_d, est = gix.search_stages(q, k, w, m)
    gix.set_exact_selection(False)
    np.testing.assert_array_equal(np.sort(est["cand_rows"].astype(np.int64), axis=1), np.sort(ost["cand_rows"], axis=1), err_msg="candidates (per-query kernel)")
    gix.set_rerank(B.RERANK_NONE)
    n_ids, n_d = gix.search(q, k, w, k)
    r_ids, r_d = O.search_no_rerank(oix, q, k, w)
    np.testing.assert_array_equal(n_ids, r_ids)
    np.testing.assert_array_equal(n_d, r_d)
    gix.close()


def test_first_rows_can_be_set_and_removed(B, small_indexes_mixed):
    """lorann_set_first_rows on a loaded index, off again with NULLs, dropped together with the column step sizes,
    and its refusals (no column step sizes, one array of two, a non-finite value)."""
    wl, ixm, corpus, queries = small_indexes_mixed["cos_P"]
    a = ixm.numpy()
    cols = {k: v for k, v in a.items() if k not in ("first_row_A", "first_row_B")}
    plain = {k: v for k, v in cols.items() if k not in ("scale_A_columns", "scale_B_points")}
    gix = B.Index(**plain)
    with pytest.raises(B.LorannError) as ei:
        gix.set_first_rows(a["first_row_A"], a["first_row_B"])              # needs the column-wise step sizes
    assert ei.value.code == B.LORANN_E_INVAL
    gix.set_column_scales(a["scale_A_columns"], a["scale_B_points"])
    c_ids, c_d = gix.search(queries, wl.k, wl.w, wl.m)                      # the codes read without the float rows
    oc_ids, oc_d = O.search(O.OracleIndex(cols), queries, wl.k, wl.w, wl.m)
    assert_topk_equal(c_ids, c_d, oc_ids, oc_d, "column-wise reading")
    gix.set_first_rows(torch.from_numpy(a["first_row_A"]).cuda(), a["first_row_B"])      # device and host pointers
    m_ids, m_d, mst = gix.search_stages(queries, wl.k, wl.w, wl.m)
    om_ids, om_d, ost = O.search(O.OracleIndex(a), queries, wl.k, wl.w, wl.m, stages=True)
    np.testing.assert_array_equal(mst["rho0"], ost["rho0"])
    np.testing.assert_array_equal(mst["z"], ost["z"])
    assert_topk_equal(m_ids, m_d, om_ids, om_d, "mixed-precision reading")
    bad = a["first_row_B"].copy(); bad[7] = np.inf
    for fa, fb in [(a["first_row_A"], None), (None, a["first_row_B"]), (a["first_row_A"], bad)]:
        with pytest.raises(B.LorannError) as ei:
            gix.set_first_rows(fa, fb)
        assert ei.value.code == B.LORANN_E_INVAL
    k_ids, k_d = gix.search(queries, wl.k, wl.w, wl.m)                      # a refused call changes nothing
    np.testing.assert_array_equal(k_ids, m_ids)
    gix.set_first_rows(None, None)
    b_ids, b_d = gix.search(queries, wl.k, wl.w, wl.m)
    np.testing.assert_array_equal(b_ids, c_ids)
    np.testing.assert_array_equal(b_d, c_d)
    gix.set_first_rows(a["first_row_A"], a["first_row_B"])
    gix.set_column_scales(None, None)                                       # takes the float rows with it
    p_ids, p_d, pst = gix.search_stages(queries, wl.k, wl.w, wl.m)
    o_ids, o_d = O.search(O.OracleIndex(plain), queries, wl.k, wl.w, wl.m)
    assert not pst["rho0"].any()
    assert_topk_equal(p_ids, p_d, o_ids, o_d, "per-cluster reading")
    gix.close()


def test_lanes_overlap_searches_with_identical_results(B, small_indexes):
    """lorann_search_lane: batches of different sizes enqueued round-robin on all lanes (each lane reused several
    times, so its workspace is recycled while other lanes are busy), joined onto the index's stream and synchronised
    once: every batch must equal the synchronous search; the queries are produced on the index's stream right before
    the call (the lane must wait for them); bad lanes and host pointers are refused."""
    wl, ix, corpus, queries = small_indexes["l2_P_norms"]
    gix = B.Index.from_arrays(ix.to("cuda"))
    gix.use_torch_stream()
    k, w, m = wl.k, wl.w, wl.m
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(21)
    sizes = [33, 200, 7, 129, 64, 1, 40, 180, 5, 77]
    picks = [rng.choice(queries.shape[0], size=n, replace=True) for n in sizes]
    host_q = [torch.from_numpy(queries[p]) for p in picks]
    outs = [(torch.empty((n, k), dtype=torch.int64, device=dev), torch.empty((n, k), dtype=torch.float32, device=dev)) for n in sizes]
    bufs = [torch.zeros((n, queries.shape[1]), dtype=torch.float32, device=dev) for n in sizes]
    gix.profile_enable(True)
    for i, (hq, o, b) in enumerate(zip(host_q, outs, bufs)):
        b.copy_(hq.to(dev) * 0.5).mul_(2.0)              # produced by kernels on the index's stream just before the call
        gix.search(b, k, w, m, out=o, lane=i % B.LANES)
    for l in range(B.LANES):
        gix.lane_join(l)
    torch.cuda.synchronize()
    assert gix.profile_get()["rerank"][1] == len(sizes)
    gix.profile_enable(False)
    for hq, o in zip(host_q, outs):
        s_ids, s_d = gix.search(hq.to(dev), k, w, m)
        np.testing.assert_array_equal(o[0].cpu().numpy(), s_ids.cpu().numpy())
        np.testing.assert_array_equal(o[1].cpu().numpy(), s_d.cpu().numpy())
    # the oracle agrees with what the lanes returned
    o_ids, o_d = O.search(O.OracleIndex(ix.numpy()), queries[picks[1]], k, w, m)
    assert_topk_equal(outs[1][0].cpu().numpy(), outs[1][1].cpu().numpy(), o_ids, o_d, "lane 1")
    for bad in (-1, B.LANES):
        with pytest.raises(B.LorannError):
            gix.search(bufs[0], k, w, m, out=outs[0], lane=bad)
        with pytest.raises(B.LorannError):
            gix.lane_join(bad)
    with pytest.raises(B.LorannError):
        gix.search(queries[:4], k, w, m, lane=1)
    # gathers of different lanes allowed to overlap: same results
    gix.set_gather_turns(False)
    for i, (b, o) in enumerate(zip(bufs, outs)):
        o[0].zero_(); o[1].zero_()
        gix.search(b, k, w, m, out=o, lane=(i + 1) % B.LANES)
    for l in range(B.LANES):
        gix.lane_join(l)
    torch.cuda.synchronize()
    gix.set_gather_turns(True)
    for hq, o in zip(host_q, outs):
        s_ids, s_d = gix.search(hq.to(dev), k, w, m)
        np.testing.assert_array_equal(o[0].cpu().numpy(), s_ids.cpu().numpy())
        np.testing.assert_array_equal(o[1].cpu().numpy(), s_d.cpu().numpy())
    # mode changes wait for the lanes: enqueue, switch, and the earlier results are those of the earlier mode
    gix.search(bufs[1], k, w, m, out=outs[1], lane=2)
    gix.set_rerank(B.RERANK_NONE)
    gix.set_rerank(B.RERANK_F32)
    s_ids, s_d = gix.search(bufs[1], k, w, m)
    np.testing.assert_array_equal(outs[1][0].cpu().numpy(), s_ids.cpu().numpy())
    gix.close()


@pytest.mark.parametrize("L", [40, 1500, 5000])
@pytest.mark.parametrize("metric", [0, 1])
def test_routing_by_screening_worst_case_rounding(B, L, metric):
    """bfloat16 keeps 8 significant bits, so 1 + 2^-8 rounds (ties to even) down to 1 and anything just above it up
    to 1 + 2^-7: a relative error of 2^-8 per operand, 2^-7 per product.  Centroid A and the query agree on 512
    coordinates where both round down, centroid B and the query on 511 coordinates where both round up: A is the
    nearest centroid (inner product 516.008 against 515.016) but the bfloat16 scores say 512.0 against 519.016, a
    gap of 7.0 = 0.0096 |q| |mu|.  The short list must still contain A (an error bound built on a unit roundoff
    of 2^-9 drops it)."""
    rng = np.random.default_rng(90 + L + metric)
    d = 1024
    lo, hi = np.float32(1 + 2.0 ** -8), np.float32(1 + 2.0 ** -8 + 2.0 ** -16)
    cent = (0.01 * rng.normal(size=(L, d))).astype(np.float32)
    ia, ib = 3, L - 5
    cent[ia] = 0.0; cent[ia, :512] = lo
    cent[ib] = 0.0; cent[ib, 512:1023] = hi
    q = np.zeros((6, d), np.float32)
    q[:, :512] = lo
    q[:, 512:1023] = hi
    q[1] *= np.float32(0.5)                           # powers of two keep the ties
    q[2] *= np.float32(8.0)
    q[3, 1023] = 0.25
    q[4, :512] = hi; q[4, 512:1023] = lo              # mixed: the query rounds up where A rounds down and vice versa
    q[5] = q[0]; q[5, 0] = 0.0
    sizes = rng.integers(1, 4, size=L)
    n = int(sizes.sum())
    off = np.zeros(L + 1, np.int64)
    np.cumsum(sizes, out=off[1:])
    ix = dict(metric=metric, n=n, d=d, dp=d, r=8, L=L, centroids=cent, P=None,
              A=rng.integers(-127, 128, size=(L, 8, d)).astype(np.int8), B=rng.integers(-127, 128, size=(n, 8)).astype(np.int8),
              scale_A=np.full(L, 0.01, np.float32), scale_B=np.full(L, 0.01, np.float32), cluster_offsets=off,
              corpus=rng.normal(size=(n, d)).astype(np.float32), ids=None)
    gix = B.Index(**ix)
    oix = O.OracleIndex(ix)
    for w in (1, 2, 3):
        ost = O.search(oix, q, 1, w, 4, stages=True)[2]
        gst = gix.search_stages(q, 1, w, 4)[2]
        np.testing.assert_array_equal(gst["sel"], ost["sel"], err_msg=f"w={w}")
    assert O.search(oix, q[:1], 1, 1, 4, stages=True)[2]["sel"][0, 0] == ia       # A is the nearest centroid of the first query
    gix.close()


def test_routing_with_a_score_matrix_beyond_the_caches(B):
    """9000 queries x 8192 clusters: the approximate score matrix (295 MB) takes the streaming stores / loads; the
    selected clusters of sampled queries must equal the oracle's."""
    rng = np.random.default_rng(44)
    L, d, nq = 8192, 32, 9000
    n = 2 * L
    ix = dict(metric=1, n=n, d=d, dp=d, r=8, L=L, centroids=rng.normal(size=(L, d)).astype(np.float32), P=None,
              A=rng.integers(-127, 128, size=(L, 8, d)).astype(np.int8), B=rng.integers(-127, 128, size=(n, 8)).astype(np.int8),
              scale_A=np.full(L, 0.01, np.float32), scale_B=np.full(L, 0.01, np.float32),
              cluster_offsets=np.arange(L + 1, dtype=np.int64) * 2, corpus=rng.normal(size=(n, d)).astype(np.float32), ids=None)
    q = rng.normal(size=(nq, d)).astype(np.float32)
    gix = B.Index(**ix)
    gst = gix.search_stages(q, 5, 24, 20)[2]
    pick = np.concatenate([np.arange(0, 60), np.arange(4470, 4530), np.arange(nq - 60, nq)])
    ost = O.search(O.OracleIndex(ix), q[pick], 5, 24, 20, stages=True)[2]
    np.testing.assert_array_equal(gst["sel"][pick], ost["sel"])
    np.testing.assert_array_equal(gst["z"][pick], ost["z"])
    gix.close()


@pytest.mark.parametrize("L,metric", [(900, 0), (3000, 1), (6000, 2), (16384, 0)])
def test_query_codes_when_the_selection_kernel_quantizes(B, L, metric):
    """With a projection and routing by screening the query is quantized inside the cluster-selection kernel (one
    wavefront or one block per query) and the projection writes the bfloat16 copy: projected queries, codes, step
    sizes and selected clusters bit-exact, an all-zero query included."""
    rng = np.random.default_rng(3000 + L)
    n = 2 * L + 17
    ix = _random_index(rng, n=n, d=48, L=L, r=8, metric=metric, dp=32)
    q = rng.normal(size=(70, 48)).astype(np.float32) * np.exp(rng.normal(size=(70, 1)) * 2).astype(np.float32)
    q[5] = 0.0
    gix = B.Index(**ix)
    o_ids, o_d, ost = O.search(O.OracleIndex(ix), q, 5, 12, 30, stages=True)
    g_ids, g_d, gst = gix.search_stages(q, 5, 12, 30)
    for key in ("qproj", "q8", "dx", "sel", "z", "sigma"):
        np.testing.assert_array_equal(gst[key], ost[key], err_msg=key)
    assert_topk_equal(g_ids, g_d, o_ids, o_d, f"L={L}")
    gix.close()


@pytest.mark.parametrize("seed", list(range(24)))
def test_randomized_configurations(B, seed):
    """Seeded random shapes and parameters - metric, d, d' (with and without projection), rank, cluster count and
    sizes (empty clusters included), w, m, k, per-cluster or column-wise step sizes, re-rank mode, batch size - each
    compared with the oracle: selected clusters, re-quantized vectors, pair scales and candidate sets bit-exact,
    results to the usual bar."""
    _randomized(B, np.random.default_rng(7000 + seed), f"seed={seed}", mixed=False)


@pytest.mark.parametrize("seed", list(range(12)))
def test_randomized_configurations_mixed_precision(B, seed):
    """The same random shapes with the mixed-precision decomposition switched on (float first rows of every size)."""
    _randomized(B, np.random.default_rng(11000 + seed), f"mixed seed={seed}", mixed=True)


def _randomized(B, rng, tag, mixed):
    metric = int(rng.integers(0, 3))
    dp = int(rng.choice([16, 32, 48, 64, 128, 256]))
    d = dp if rng.random() < 0.3 else int(dp + rng.integers(1, 200))
    r = int(rng.choice([8, 16, 24, 32, 40, 64]))
    L = int(rng.choice([1, 2, 7, 33, 150, 700, 1300, 2500]))
    n = int(max(L, rng.integers(L, 40 * L + 50)))
    nq = int(rng.choice([1, 3, 17, 64, 130, 400]))
    w = int(rng.integers(1, min(L, 40) + 1))
    m = int(rng.choice([1, 5, 30, 100, 256, 300, 600]))
    k = int(rng.integers(1, min(m, 80) + 1))
    ix = _random_index(rng, n=max(n, 2), d=d, L=L, r=r, metric=metric, dp=dp) if L > 1 else None
    if ix is None:      # a single cluster
        n = max(n, 2)
        corpus = rng.normal(size=(n, d)).astype(np.float32)
        if metric == 2:
            corpus /= np.linalg.norm(corpus, axis=1, keepdims=True)
        P = None if dp == d else np.linalg.qr(rng.normal(size=(d, d)))[0][:, :dp].astype(np.float32)
        ix = dict(metric=metric, n=n, d=d, dp=dp, r=r, L=1, centroids=rng.normal(size=(1, dp)).astype(np.float32), P=P,
                  A=rng.integers(-127, 128, size=(1, r, dp)).astype(np.int8), B=rng.integers(-127, 128, size=(n, r)).astype(np.int8),
                  scale_A=np.array([0.03], np.float32), scale_B=np.array([0.05], np.float32),
                  cluster_offsets=np.array([0, n], np.int64), corpus=corpus, ids=None)
    n = ix["n"]
    if L > 3:           # some empty clusters
        off = ix["cluster_offsets"].copy()
        for c in rng.choice(np.arange(1, L), size=min(3, L - 1), replace=False):
            off[c] = off[c - 1]
        ix["cluster_offsets"] = np.maximum.accumulate(off)
    if rng.random() < 0.4:
        ix["scale_A_columns"] = (10.0 ** rng.uniform(-3, 0, size=(L, r))).astype(np.float32)
        ix["scale_B_points"] = (10.0 ** rng.uniform(-3, 0, size=n)).astype(np.float32)
    q = rng.normal(size=(nq, d)).astype(np.float32)
    mode = int(rng.choice([B.RERANK_F32, B.RERANK_F32, B.RERANK_F16, B.RERANK_NONE]))
    if mixed:
        if "scale_A_columns" not in ix:
            ix["scale_A_columns"] = (10.0 ** rng.uniform(-3, 0, size=(L, r))).astype(np.float32)
            ix["scale_B_points"] = (10.0 ** rng.uniform(-3, 0, size=n)).astype(np.float32)
        ix["first_row_A"] = (rng.normal(size=(L, r)) * 10.0 ** rng.uniform(-2, 1, size=(L, 1))).astype(np.float32)
        ix["first_row_B"] = (rng.normal(size=n) * 10.0 ** rng.uniform(-2, 1, size=n)).astype(np.float32)
    what = f"{tag} metric={metric} d={d} dp={dp} r={r} L={L} n={n} nq={nq} w={w} m={m} k={k} cols={'scale_A_columns' in ix} mode={mode}"
    gix = B.Index(**ix)
    gix.set_rerank(mode)
    oracle_ix = O.with_half_precision_corpus(ix) if mode == B.RERANK_F16 else ix
    oix = O.OracleIndex(oracle_ix)
    if mode == B.RERANK_NONE:
        o_ids, o_d = O.search_no_rerank(oix, q, k, w)
        g_ids, g_d = gix.search(q, k, w, m)
        np.testing.assert_array_equal(g_ids, o_ids, err_msg=what)
        np.testing.assert_array_equal(g_d, o_d, err_msg=what)
    else:
        o_ids, o_d, ost = O.search(oix, q, k, w, m, stages=True)
        g_ids, g_d, gst = gix.search_stages(q, k, w, m)
        for key in ("q8", "dx", "sel", "z", "sigma", "rho0"):
            np.testing.assert_array_equal(gst[key], ost[key], err_msg=f"{key}: {what}")
        np.testing.assert_array_equal(np.sort(gst["cand_rows"].astype(np.int64), axis=1), np.sort(ost["cand_rows"], axis=1), err_msg=what)
        if "pmax" in gst:
            np.testing.assert_array_equal(gst["pmax"], ost["pair_best"], err_msg=f"per-pair best scores: {what}")
        # k can reach most of the scored points here, so the results include inner products that cancel to almost
        # nothing: those carry the float rounding of their terms (bound d 2^-24 |q| |x|) whatever their own size
        rr = oracle_ix.get("rerank_corpus")
        assert_topk_equal(g_ids, g_d, o_ids, o_d, what, abs_tol=rounding_abs_tol(q, ix["corpus"], metric),
                          exact=oracle_distance_of(ix, q, rerank_corpus=rr))
    gix.close()


@pytest.mark.parametrize("nq", [1, 2, 15, 16, 17, 32, 33, 40])
def test_small_batches_take_the_small_projection(B, small_indexes, nq):
    """Batches of up to 512 queries are projected by the one-wavefront-per-output-column kernel - one query per
    wavefront up to 32 queries, 16 per wavefront beyond (the workload has 40 queries): projected queries, codes and
    everything after them bit-exact."""
    wl, ix, corpus, queries = small_indexes["cos_P"]
    a = ix.numpy()
    q = queries[:nq]
    o_ids, o_d, ost = O.search(O.OracleIndex(a), q, wl.k, wl.w, wl.m, stages=True)
    gix = B.Index.from_arrays(ix.to("cuda"))
    g_ids, g_d, gst = gix.search_stages(q, wl.k, wl.w, wl.m)
    for key in ("qproj", "q8", "dx", "sel", "z", "sigma"):
        np.testing.assert_array_equal(gst[key], ost[key], err_msg=key)
    assert_topk_equal(g_ids, g_d, o_ids, o_d, f"nq={nq}")
    gix.close()


@pytest.mark.parametrize("nq,d,dp", [(513, 48, 32), (700, 50, 32), (2000, 200, 64), (1500, 333, 256)])
def test_batches_beyond_the_small_projection_use_the_matrix_cores(B, nq, d, dp):
    """More than 512 queries are projected on the fp64 matrix cores (rows that are and are not a multiple of four
    floats, both tile heights): projected queries, codes, step sizes and selected clusters bit-exact."""
    rng = np.random.default_rng(nq + d)
    ix = _random_index(rng, n=900, d=d, L=20, r=8, metric=int(nq % 3), dp=dp)
    q = rng.normal(size=(nq, d)).astype(np.float32)
    gix = B.Index(**ix)
    o_ids, o_d, ost = O.search(O.OracleIndex(ix), q, 5, 4, 30, stages=True)
    g_ids, g_d, gst = gix.search_stages(q, 5, 4, 30)
    for key in ("qproj", "q8", "dx", "sel", "z", "sigma"):
        np.testing.assert_array_equal(gst[key], ost[key], err_msg=key)
    assert_topk_equal(g_ids, g_d, o_ids, o_d, f"nq={nq}", abs_tol=rounding_abs_tol(q, ix["corpus"], ix["metric"]),
                      exact=oracle_distance_of(ix, q))
    gix.close()
