"""The seeded input generators: determinism, shapes, and the index builder against the numpy RRR fit."""
import numpy as np
import torch

from oracle import rrr_fit as F
from paper_2410_18926_amd.synth import build_index, get_workload, make_dataset
from paper_2410_18926_amd.synth.workloads import IP, L2


def test_dataset_is_seeded_and_shaped(small_workloads):
    wl = small_workloads["ip_P"]
    c1, q1 = make_dataset(wl)
    c2, q2 = make_dataset(wl)
    assert torch.equal(c1, c2) and torch.equal(q1, q2)
    assert c1.shape == (wl.n, wl.d) and q1.shape == (wl.nq, wl.d) and c1.dtype == torch.float32
    np.testing.assert_allclose(c1.norm(dim=1).numpy(), 1.0, rtol=1e-5)
    wl4 = small_workloads["l2_P_norms"]
    c4, _ = make_dataset(wl4)
    ln = torch.log(c4.norm(dim=1))
    assert abs(float(ln.mean())) < 0.05 and abs(float(ln.std()) - 0.5) < 0.05     # LogNormal(0, 0.5) norms


def test_tiny_workload_matches_its_description():
    wl = get_workload("tiny")
    assert (wl.n, wl.d, wl.nq, wl.G, wl.L, wl.dp, wl.r, wl.w, wl.m, wl.k) == (20000, 128, 1000, 64, 64, 128, 32, 8, 100, 10)
    assert wl.metric == L2 and wl.n_train == 5000
    c2 = get_workload("embed-ip")
    assert (c2.n, c2.d, c2.nq, c2.G, c2.L, c2.dp, c2.r, c2.w, c2.m, c2.metric) == (1000000, 768, 10000, 4096, 1024, 256, 32, 32, 200, IP)


def test_index_layout_and_partition(small_indexes):
    for name, (wl, ix, corpus, queries) in small_indexes.items():
        a = ix.numpy()
        off = a["cluster_offsets"]
        assert off[0] == 0 and off[-1] == wl.n and np.all(np.diff(off) >= 0)
        assert sorted(a["ids"].tolist()) == list(range(wl.n))                    # a partition: every point once
        np.testing.assert_array_equal(corpus[a["ids"]], a["corpus"])
        assert a["A"].shape == (wl.L, wl.r, wl.dp) and a["B"].shape == (wl.n, wl.r)
        assert (a["P"] is None) == (wl.dp == wl.d)
        if a["P"] is not None:                                                   # orthonormal columns
            np.testing.assert_allclose(a["P"].T.astype(np.float64) @ a["P"].astype(np.float64), np.eye(wl.dp), atol=1e-5)
        # every point sits in the cluster of its nearest centroid (in the projected space)
        xp = a["corpus"] if a["P"] is None else a["corpus"] @ a["P"]
        ip = xp.astype(np.float64) @ a["centroids"].astype(np.float64).T
        g = (a["centroids"].astype(np.float64) ** 2).sum(1)[None] - 2 * ip if wl.metric == L2 else -ip
        lab = np.repeat(np.arange(wl.L), np.diff(off))
        best = g.min(1)
        assert np.mean(g[np.arange(wl.n), lab] <= best + 1e-4 * np.abs(best) + 1e-5) > 0.999
        # absmax codes: each non-empty cluster uses the full code range
        for c in range(wl.L):
            if off[c + 1] > off[c] and a["scale_B"][c] > 0:
                assert np.abs(a["B"][off[c]:off[c + 1]].astype(int)).max() == 127
                assert np.abs(a["A"][c].astype(int)).max() == 127


def test_builder_fit_matches_numpy_rrr(small_workloads):
    """Exact-SVD, unrotated builder == oracle/rrr_fit.py on every cluster: same rank-r coefficient matrix
    beta = A B (the factors themselves are unique only up to an r x r rotation/sign)."""
    for key in ("l2_noP", "ip_P"):
        wl = small_workloads[key]
        corpus, _ = make_dataset(wl)
        train = corpus[: wl.n_train]
        ix = build_index(corpus, wl, exact_svd=True, rotate=False, keep_float=True, train=train)
        a = ix.numpy()
        off = a["cluster_offsets"]
        W = None if a["P"] is None else a["P"].astype(np.float64)
        # local training sets: training points with the cluster among their w_train nearest centroids
        tp = train.numpy() if W is None else train.numpy().astype(np.float64) @ W
        ip = tp.astype(np.float64) @ a["centroids"].astype(np.float64).T
        g = (a["centroids"].astype(np.float64) ** 2).sum(1)[None] - 2 * ip if wl.metric == L2 else -ip
        routed = np.argsort(g, axis=1, kind="stable")[:, : wl.w_train]
        checked = 0
        for c in range(wl.L):
            m_c = off[c + 1] - off[c]
            X = train.numpy()[np.any(routed == c, axis=1)]
            if m_c <= wl.r or X.shape[0] < max(wl.dp, wl.r) + 5:
                continue
            C = a["corpus"][off[c]:off[c + 1]]
            A_ref, B_ref = F.rrr_fit(X, C, wl.r, W)
            beta = a["A_f32"][c].astype(np.float64).T @ a["B_f32"][off[c]:off[c + 1]].astype(np.float64).T
            beta_ref = A_ref @ B_ref
            assert np.linalg.norm(beta - beta_ref) <= 2e-3 * np.linalg.norm(beta_ref), (key, c)
            # 8-bit codes are the absmax quantization of the float factors
            codes, delta = F.absmax_quantize(a["B_f32"][off[c]:off[c + 1]])
            np.testing.assert_array_equal(codes, a["B"][off[c]:off[c + 1]])
            assert abs(delta - a["scale_B"][c]) <= 1e-6 * delta
            codes, delta = F.absmax_quantize(a["A_f32"][c])
            np.testing.assert_array_equal(codes, a["A"][c])
            checked += 1
        assert checked >= 3
