"""The error bound behind routing by screening (CPU check of the mathematics; the GPU kernels rely on it).

Approximate centroid scores come from operands rounded to bfloat16 with float accumulation; the library keeps
every cluster whose approximate value is within 2 eps of the w-th smallest, with
eps = |dq| max|mu| + |qb| max|dmu| + d' 2^-23 |qb| (max|mu| + max|dmu|)  (dq, dmu: the actual rounding errors of the
query and of the centroids, qb the rounded query; doubled plus a float-rounding term for the Euclidean form; every
norm rounded up by 1e-3).  Here the inequality |approximate - exact| <= eps is checked on
seeded inputs of several scales, including the worst case of bfloat16 (8 significant bits: every element of both
vectors sits on, or just beside, the midpoint 1 + 2^-8 between two neighbours, all errors of one sign), with
bfloat16 emulated by torch on the CPU.
"""
import numpy as np
import torch

K_SCREEN_ACC = 2.0 ** -23   # must equal kScreenAcc in csrc/screen.hpp


def _bf16(x):
    return torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()


def test_constant_matches_the_kernel_source():
    import pathlib, re
    src = (pathlib.Path(__file__).resolve().parents[1] / "paper_2410_18926_amd" / "csrc" / "screen.hpp").read_text()
    assert abs(float(re.search(r"kScreenAcc\s*=\s*([0-9.e-]+)f", src).group(1)) - K_SCREEN_ACC) < 1e-13
    assert "qe * mu_max + qb * dmu_max + (float)dp * kScreenAcc * qb * (mu_max + dmu_max)" in src


def _eps_ip(q, c):
    """The library's bound for every query of q against the centroid set c (float64 here; the kernel rounds up)."""
    qb, cb = _bf16(q).astype(np.float64), _bf16(c).astype(np.float64)
    qe = np.linalg.norm(q.astype(np.float64) - qb, axis=1) * 1.001
    qbn = np.linalg.norm(qb, axis=1) * 1.001
    mu_max = np.linalg.norm(c.astype(np.float64), axis=1).max()
    dmu_max = np.linalg.norm(c.astype(np.float64) - cb, axis=1).max()
    return (qe * mu_max + qbn * dmu_max + q.shape[1] * K_SCREEN_ACC * qbn * (mu_max + dmu_max)) * 1.001


def test_bf16_inner_product_error_is_within_the_bound():
    rng = np.random.default_rng(5)
    for dp in (16, 64, 256, 1024):
        for scale_q, scale_c in ((1.0, 1.0), (1e-3, 40.0), (300.0, 1e-2)):
            q = (scale_q * rng.normal(size=(64, dp))).astype(np.float32)
            c = (scale_c * rng.normal(size=(200, dp))).astype(np.float32)
            # worst case for round-to-nearest: mantissas on / just below the midpoint between two bfloat16 values
            # (1 and 1 + 2^-7), rows 0-3 with every product positive so that all errors add up; rows 4-7 just
            # above the midpoint (rounded up)
            bad = (np.float32(1.0) + np.float32(2.0 ** -8) * np.float32(0.9999)) * np.sign(rng.normal(size=(8, dp))).astype(np.float32)
            bad[:2] = np.float32(1.0) + np.float32(2.0 ** -8)              # exact ties: to even, i.e. down to 1
            bad[2:4] = np.abs(bad[2:4])
            bad[4:] = (np.float32(1.0) + np.float32(2.0 ** -8) * np.float32(1.0001)) * np.sign(bad[4:])
            q[:8] = scale_q * bad
            c[:8] = scale_c * np.abs(bad)
            if scale_q == 1.0 and scale_c == 1.0:                          # scales that are powers of two keep the ties
                worst = np.abs(_bf16(q[:2]).astype(np.float64) @ _bf16(c[:2]).T.astype(np.float64) - q[:2].astype(np.float64) @ c[:2].astype(np.float64).T)
                rel = worst / (np.linalg.norm(q[:2].astype(np.float64), axis=1)[:, None] * np.linalg.norm(c[:2].astype(np.float64), axis=1)[None, :])
                assert rel.max() > 0.0077, "the worst case is not exercised"   # 2^-7 + 2^-16 over (1 + 2^-8)^2
            exact = q.astype(np.float64) @ c.astype(np.float64).T
            approx = (_bf16(q) @ _bf16(c).T).astype(np.float64)           # float accumulation
            eps_ip = _eps_ip(q, c)
            assert np.all(np.abs(approx - exact) <= eps_ip[:, None]), (dp, scale_q, scale_c, float(np.max(np.abs(approx - exact) / eps_ip[:, None])))
            # the bound adapts: for the ordinary rows it is well below the worst case 2^-7 |q| |mu|
            typical = eps_ip[8:] / (np.linalg.norm(q[8:].astype(np.float64), axis=1) * np.linalg.norm(c.astype(np.float64), axis=1).max())
            assert typical.max() < 0.0065
            # Euclidean form: |mu|^2 - 2 ip with the norm rounded to float
            nrm = (c.astype(np.float64) ** 2).sum(1)
            g = nrm[None, :] - 2.0 * exact
            g_hat = (nrm.astype(np.float32)[None, :] - np.float32(2.0) * approx.astype(np.float32)).astype(np.float64)
            qn, mu_max, nrm_max = np.linalg.norm(q.astype(np.float64), axis=1), np.sqrt(nrm.max()), nrm.max()
            eps = 2.0 * eps_ip + 2.4e-7 * (nrm_max + 2.0 * qn * mu_max)
            assert np.all(np.abs(g_hat - g) <= eps[:, None])


def test_the_list_contains_the_exact_w_best():
    """The selection rule itself, in numpy: everything within 2 eps of the w-th smallest approximate value."""
    rng = np.random.default_rng(6)
    dp, L, w = 64, 2000, 48
    c = rng.normal(size=(L, dp)).astype(np.float32)
    c /= np.linalg.norm(c, axis=1, keepdims=True)
    c[100:400] = c[100] * (1.0 + 1e-6 * rng.normal(size=(300, 1))).astype(np.float32)     # a crowd of near-equal scores
    q = (c[100][None, :] + 0.05 * rng.normal(size=(32, dp))).astype(np.float32)
    exact = (-(q.astype(np.float64) @ c.astype(np.float64).T)).astype(np.float32)
    approx = -(_bf16(q) @ _bf16(c).T)
    eps = _eps_ip(q, c)
    for i in range(q.shape[0]):
        best = np.argsort(exact[i], kind="stable")[:w]
        gw = np.sort(approx[i])[w - 1]
        listed = approx[i] <= gw + 2.0 * eps[i]
        assert listed[best].all()
        assert listed.sum() >= w


def test_subset_minima_bound_and_lists_give_the_same_list():
    """The route that never forms the full row of approximate values: the w-th smallest of the minima of 256 disjoint
    subsets of the clusters bounds the w-th smallest approximate value from above, so the entries at or below that
    bound + 2 eps - even when they come from a second evaluation whose float additions ran in another order, i.e. differ
    from the first within eps - contain the w-th smallest approximate value and the whole final list of the rule above;
    the final list built from them is the list built from the full row."""
    rng = np.random.default_rng(8)
    dp, L, w, S = 64, 5000, 64, 256
    c = rng.normal(size=(L, dp)).astype(np.float32)
    c /= np.linalg.norm(c, axis=1, keepdims=True)
    c[700:1000] = c[700] * (1.0 + 1e-6 * rng.normal(size=(300, 1))).astype(np.float32)
    q = (c[700][None, :] + 0.05 * rng.normal(size=(24, dp))).astype(np.float32)
    q[12:] = rng.normal(size=(12, dp)).astype(np.float32)
    exact = (-(q.astype(np.float64) @ c.astype(np.float64).T)).astype(np.float32)
    qb, cb = _bf16(q), _bf16(c)
    first = -(qb @ cb.T)                                                   # float accumulation, one order
    second = -np.add.reduce((qb[:, None, ::-1] * cb[None, :, ::-1]).astype(np.float32), axis=2, dtype=np.float32)   # another order
    eps = _eps_ip(q, c)
    assert np.all(np.abs(second.astype(np.float64) - exact) <= eps[:, None])
    # subsets as the kernel forms them: clusters with equal (l mod 64 row pattern, run of tiles) - any disjoint partition will do
    subset = (np.arange(L) % 32) + 32 * np.minimum((np.arange(L) // 64) // ((L // 64 + 8) // 8), 7)
    assert subset.max() < S
    for i in range(q.shape[0]):
        mins = np.full(S, np.inf, np.float32)
        np.minimum.at(mins, subset, first[i])
        bound = np.sort(mins)[w - 1]
        assert bound >= np.sort(first[i])[w - 1]
        thr = bound + 2.0 * eps[i]
        listed = second[i] <= thr
        best = np.argsort(exact[i], kind="stable")[:w]
        assert listed[best].all() and listed.sum() >= w
        gw_list = np.sort(second[i][listed])[w - 1]
        assert gw_list == np.sort(second[i])[w - 1]                        # the w-th smallest approximate value is in the list
        final_from_list = np.flatnonzero(listed)[second[i][listed] <= gw_list + 2.0 * eps[i]]
        final_from_row = np.flatnonzero(second[i] <= gw_list + 2.0 * eps[i])
        np.testing.assert_array_equal(final_from_list, final_from_row)
        assert np.isin(best, final_from_list).all()
