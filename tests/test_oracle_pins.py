"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU, no HIP library).

Each test names the passage it checks.  Independent evidence used: numpy/Python-integer re-computation,
library eigh/SVD, brute force, closed-form error bounds.
"""
from fractions import Fraction

import numpy as np
import pytest

from oracle import oracle as O
from oracle import rrr_fit as F

IP, L2, COS = 0, 1, 2
rng = np.random.default_rng(20241018)


# ------------------------------------------------------------------ Sec. 3.2: the score model
def _cluster(n_l=90, m_l=70, d=24, seed=0):
    g = np.random.default_rng(seed)
    scales = np.linspace(3.0, 0.3, d)                  # distinct spectrum => unique leading subspaces
    C = g.normal(size=(m_l, d)) * scales + 0.5
    X = g.normal(size=(n_l, d)) * scales[::-1] * 0.7 + 0.2
    return X, C


def test_full_rank_reproduces_exact_inner_products():
    """Sec. 3.2: the unconstrained least-squares solution beta = C^T gives y = x^T C^T.  At r = d the
    factorised prediction (x^T A) B must equal the exact inner products."""
    X, C = _cluster()
    d = C.shape[1]
    A, B = F.rrr_fit(X, C, r=d)
    for _ in range(5):
        x = rng.normal(size=d)
        y = O.rrr_predict_f64(x, A, B)
        np.testing.assert_allclose(y, C @ x, rtol=1e-8, atol=1e-9)


def test_theorem1_training_on_cluster_equals_projected_inner_products():
    """Appendix A, Theorem 1: with X = C the RRR prediction equals the inner products of query and cluster
    points after projecting both on the first r eigenvectors of C^T C (library eigh as the reference)."""
    _, C = _cluster(seed=3)
    r = 6
    A, B = F.rrr_fit(C, C, r=r)
    evals, evecs = np.linalg.eigh(C.T @ C)
    Wr = evecs[:, np.argsort(evals)[::-1][:r]]
    for _ in range(5):
        x = rng.normal(size=C.shape[1])
        y = O.rrr_predict_f64(x, A, B)
        np.testing.assert_allclose(y, (Wr.T @ x) @ (C @ Wr).T, rtol=1e-7, atol=1e-8)


def test_rrr_beats_other_rank_r_factorisations_on_training_loss():
    """Sec. 3.2 / Appendix A: beta_RRR minimises |Y - X beta|_F over rank-r matrices; in particular it is
    no worse than the truncated SVD of C^T and than perturbed rank-r candidates when X != C."""
    X, C = _cluster(seed=5)
    r = 5
    A, B = F.rrr_fit(X, C, r=r)
    Y = X @ C.T
    loss = np.linalg.norm(Y - X @ (A @ B)) ** 2
    U, S, Vt = np.linalg.svd(C.T, full_matrices=False)
    beta_svd = (U[:, :r] * S[:r]) @ Vt[:r]
    assert loss <= np.linalg.norm(Y - X @ beta_svd) ** 2 * (1 + 1e-12)
    assert loss < np.linalg.norm(Y - X @ beta_svd) ** 2 * 0.999     # and strictly better here (X != C)
    for t in range(10):
        g = np.random.default_rng(t)
        cand = (A + 0.05 * g.normal(size=A.shape)) @ (B + 0.05 * g.normal(size=B.shape))
        assert loss <= np.linalg.norm(Y - X @ cand) ** 2


def test_rrr_with_dimensionality_reduction_is_least_squares_on_projected_inputs():
    """Sec. 4.1: A = (X W_s)^+ Y V_r with the TRUE inner products as outputs.  Checked through the normal
    equations (residual orthogonal to the projected inputs), V_r orthonormal, and B = V_r^T spanning the
    leading right singular subspace of Y."""
    X, C = _cluster(seed=7)
    s, r = 10, 4
    W = F.projection_matrix(X, s)
    evals = np.linalg.eigvalsh(X.T @ X)[::-1]
    np.testing.assert_allclose(np.sort(np.diag(W.T @ (X.T @ X) @ W))[::-1], evals[:s], rtol=1e-9)
    A, B = F.rrr_fit(X, C, r, W)
    assert A.shape == (s, r) and B.shape == (r, C.shape[0])
    Y = X @ C.T
    np.testing.assert_allclose(B @ B.T, np.eye(r), atol=1e-10)
    resid = Y @ B.T - (X @ W) @ A
    np.testing.assert_allclose((X @ W).T @ resid, 0, atol=1e-6)
    sv = np.linalg.svd(Y, compute_uv=False)
    np.testing.assert_allclose(np.linalg.norm(Y @ B.T) ** 2, (sv[:r] ** 2).sum(), rtol=1e-9)


# ------------------------------------------------------------------ Sec. 3.3: quantization
def test_query_quantization_properties():
    """Sec. 3.3 absmax: codes = round(127/|x|_inf * x): the largest code is +-127, every element is within
    half a step of its code, the step is |x|_inf / 127; the zero vector maps to zero codes and step 0."""
    for trial in range(50):
        qp = (rng.normal(size=64) * rng.uniform(1e-3, 1e3)).astype(np.float32)
        q8, dx = O.quantize_query(qp)
        a = np.abs(qp).max()
        assert np.abs(q8.astype(int)).max() == 127
        assert dx == np.float32(a) / np.float32(127)
        err = np.abs(qp.astype(np.float64) - float(dx) * q8.astype(np.float64))
        assert err.max() <= 0.5 * float(dx) * (1 + 1e-5)
        assert q8[np.argmax(np.abs(qp))] == 127 * np.sign(qp[np.argmax(np.abs(qp))])
    q8, dx = O.quantize_query(np.zeros(16, np.float32))
    assert not q8.any() and dx == 0


def test_query_quantization_rounds_half_to_even():
    """Reading of the paper's 'rounding to the nearest integer': ties go to the even code."""
    # max = 127 => multiplier exactly 1; values k + 0.5 are exact in float
    qp = np.array([127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.49], np.float32)
    q8, dx = O.quantize_query(qp)
    assert q8.tolist() == [127, 0, 2, 2, 0, -2, -2, 3] and dx == 1.0


def test_stage_a_accumulators_and_requantization_exact():
    """Sec. 3.3: r_i32 = x_i8^T A_i8 exactly (int64 matmul as reference); the re-quantized vector is
    round-half-away(127 R_j / max|R|) checked in exact rational arithmetic; codes stay within +-127."""
    for trial in range(30):
        dp, r = int(rng.integers(1, 70)), int(rng.integers(1, 40))
        q8 = rng.integers(-127, 128, size=dp).astype(np.int8)
        A_c = rng.integers(-127, 128, size=(r, dp)).astype(np.int8)
        R, z, sigma = O.stage_a(q8, A_c, 0.25, 0.5, 2.0)
        ref = A_c.astype(np.int64) @ q8.astype(np.int64)
        assert np.array_equal(R.astype(np.int64), ref)
        M = int(np.abs(ref).max())
        for j in range(r):
            if M == 0:
                assert z[j] == 0
                continue
            x = Fraction(127 * abs(int(ref[j])), M)
            expect = int(x + Fraction(1, 2))            # floor(x + 1/2): half away from zero on |.|
            assert int(z[j]) == (expect if ref[j] >= 0 else -expect)
        assert np.abs(z.astype(int)).max() == (127 if M else 0)
        # combined scale: (M/127) * dx * dA * dB; these factors are exact in binary
        assert sigma == np.float32(M / 127.0 * 0.25 * 0.5 * 2.0)


def test_stage_a_exhaustive_rounding_small():
    """All (R, M) with M <= 40: integer formula == exact rational rounding, including the .5 ties."""
    for M in range(1, 41):
        q8 = np.array([1], np.int8)
        col = np.arange(-M, M + 1)
        col = col[np.abs(col) <= 127]
        A_c = col.astype(np.int8).reshape(-1, 1)
        R, z, _ = O.stage_a(q8, A_c, 1.0, 1.0, 1.0)
        for Rj, zj in zip(R.tolist(), z.tolist()):
            e = int(Fraction(127 * abs(Rj), M) + Fraction(1, 2))
            assert zj == (e if Rj >= 0 else -e)


def test_zero_intermediate_vector():
    R, z, sigma = O.stage_a(np.zeros(8, np.int8), np.ones((4, 8), np.int8), 1.0, 1.0, 1.0)
    assert not R.any() and not z.any() and sigma == 0


def test_pair_accumulators_exact():
    """Sec. 3.3 / 4.2: y_i32 = r_i8^T B_i8 exactly, for r that is and is not a multiple of 32."""
    for r in (8, 24, 32, 48, 64):
        z = rng.integers(-127, 128, size=r).astype(np.int8)
        B_c = rng.integers(-127, 128, size=(257, r)).astype(np.int8)
        Y = O.pair_accumulators(z, B_c)
        assert np.array_equal(Y.astype(np.int64), B_c.astype(np.int64) @ z.astype(np.int64))
    # extreme values: no int32 overflow at r = 64
    z = np.full(64, -127, np.int8)
    B_c = np.full((3, 64), 127, np.int8)
    assert O.pair_accumulators(z, B_c).tolist() == [-64 * 127 * 127] * 3


def test_quantized_scores_track_float_model_within_quantization_bound(small_indexes):
    """Sec. 3.3: the 8-bit pipeline approximates (x'^T A) B.  With A, B taken at their de-quantized values
    the only errors are the query quantization (<= Delta_x / 2 per element) and the re-quantization of the
    intermediate vector (<= half a step); propagate both bounds exactly and require the oracle's score
    sigma * Y to lie inside.  A dropped or misplaced scale factor, a transposed operand or a wrong sign
    breaks this."""
    for name, (wl, ix, corpus, queries) in small_indexes.items():
        a = ix.numpy()
        oix = O.OracleIndex(a)
        ids, dists, st = O.search(oix, queries, wl.k, wl.w, wl.m, stages=True)
        for qi in range(0, len(queries), 7):
            for j in range(wl.w):
                c = int(st["sel"][qi, j])
                o0, o1 = int(a["cluster_offsets"][c]), int(a["cluster_offsets"][c + 1])
                if o1 == o0:
                    continue
                dA, dB, dx = float(a["scale_A"][c]), float(a["scale_B"][c]), float(st["dx"][qi])
                A_real = dA * a["A"][c].astype(np.float64).T            # [dp][r]
                B_real = dB * a["B"][o0:o1].astype(np.float64).T        # [r][m_c]
                qp = st["qproj"][qi].astype(np.float64)
                y_ref = (qp @ A_real) @ B_real
                err_r = 0.5 * dx * np.abs(A_real).sum(0)                 # query quantization, per j
                M = np.abs(st["R"][qi, j].astype(np.int64)).max()
                err_r = err_r + 0.5 * dx * dA * M / 127.0                # re-quantization half step
                bound = err_r @ np.abs(B_real)
                Y = O.pair_accumulators(st["z"][qi, j], a["B"][o0:o1])
                s_hat = float(st["sigma"][qi, j]) * Y.astype(np.float64)
                assert np.all(np.abs(s_hat - y_ref) <= bound * (1 + 1e-4) + 1e-6 * np.abs(y_ref).max()), name


def test_quantized_scores_approximate_true_inner_products(small_indexes):
    """End-to-end sanity of the score model on the anisotropic workloads: the estimated scores correlate
    strongly with the true inner products q.c of the scored points (Sec. 3.1: it suffices to estimate inner
    products)."""
    wl, ix, corpus, queries = small_indexes["ip_P"]
    a = ix.numpy()
    oix = O.OracleIndex(a)
    _, _, st = O.search(oix, queries, wl.k, wl.w, wl.m, stages=True)
    cors = []
    for qi in range(10):
        c = int(st["sel"][qi, 0])
        o0, o1 = int(a["cluster_offsets"][c]), int(a["cluster_offsets"][c + 1])
        if o1 - o0 < 10:
            continue
        Y = O.pair_accumulators(st["z"][qi, 0], a["B"][o0:o1]).astype(np.float64) * float(st["sigma"][qi, 0])
        true = a["corpus"][o0:o1].astype(np.float64) @ queries[qi].astype(np.float64)
        cors.append(np.corrcoef(Y, true)[0, 1])
    assert np.mean(cors) > 0.8


# ------------------------------------------------------------------ Sec. 3.3 as printed: one step size per column
def test_column_scales_stage_a_hand_example():
    """r_f32 = s (.) r_i32 with s_j = Delta_x * DeltaA_j, then absmax re-quantization (Sec. 3.3).  Numbers chosen so
    that every float operation is exact: |rho|_inf = 127 / 16, hence z = rint(16 rho) with two exact ties."""
    q8 = np.array([127, -64, 10, 0], np.int8)
    A_c = np.array([[64, 0, 0, 0],            # column 0 of A_c: R_0 = 127 * 64 = 8128
                    [0, -10, 0, 5],           # column 1:        R_1 = 640
                    [1, 2, 0, 0],             # column 2:        R_2 = 127 - 128 = -1
                    [0, 1, 0, 9]], np.int8)   # column 3:        R_3 = -64
    dx = 2.0 ** -7
    dA = np.array([2.0 ** -3, 2.0 ** -5, 2.0 ** -1, 2.0 ** -4], np.float32)
    R, z, sigma = O.stage_a_columns(q8, A_c, dx, dA)
    assert R.tolist() == [8128, 640, -1, -64]
    # rho = R * 2^-7 * dA = [127/16, 640/4096, -1/256, -64/2048]; 16 rho = [127, 2.5, -1/16, -0.5]
    assert z.tolist() == [127, 2, 0, 0]       # 2.5 -> 2 and -0.5 -> -0 (ties to even)
    assert sigma == np.float32(2.0 ** -4)
    R, z, sigma = O.stage_a_columns(np.zeros(4, np.int8), A_c, dx, dA)
    assert z.tolist() == [0, 0, 0, 0] and sigma == 0.0
    # the column step sizes are applied per column, not per row of the stored A_c^T: swap two and the codes move
    R, z, _ = O.stage_a_columns(q8, A_c, dx, dA[[1, 0, 2, 3]])
    assert z.tolist() == [127, 40, 0, -2]     # rho = [127/64, 640/1024, -1/256, -64/2048]; 64 rho = [127, 40, -1/4, -2]


def test_column_scales_requantization_is_correctly_rounded():
    """Random pairs: z_j is the integer nearest to 127 rho_j / |rho|_inf (rho from exact integer R and the float
    step sizes, evaluated with rationals), up to the float rounding of the two multiplications."""
    g = np.random.default_rng(11)
    for _ in range(50):
        dp, r = 24, 8
        q8 = g.integers(-127, 128, dp).astype(np.int8)
        A_c = g.integers(-127, 128, (r, dp)).astype(np.int8)
        dx = np.float32(g.uniform(1e-3, 1e-1))
        dA = g.uniform(1e-3, 1.0, r).astype(np.float32)
        R, z, sigma = O.stage_a_columns(q8, A_c, dx, dA)
        assert R.tolist() == [int(sum(int(a) * int(b) for a, b in zip(q8, A_c[j]))) for j in range(r)]
        rho = [Fraction(int(R[j])) * Fraction(float(dx)) * Fraction(float(dA[j])) for j in range(r)]
        M = max(abs(v) for v in rho)
        assert abs(Fraction(float(sigma)) - M / 127) <= M / 127 * Fraction(1, 2 ** 21)
        for j in range(r):
            assert abs(Fraction(int(z[j])) - 127 * rho[j] / M) <= Fraction(1, 2) + Fraction(1, 10 ** 4)
        assert max(abs(int(v)) for v in z) == 127


def test_column_scales_score_is_scale_product_then_one_fma():
    assert O.score_columns(1000, 0.375, 0.0625, IP) == np.float32(23.4375)
    assert O.score_columns(1000, 0.375, 0.0625, COS) == np.float32(23.4375)
    assert O.score_columns(1000, 0.375, 0.0625, L2, 5.5) == np.float32(41.375)
    g = np.random.default_rng(12)
    for _ in range(200):
        Y = int(g.integers(-500000, 500000))
        sg, dB, nrm = np.float32(g.uniform(1e-4, 1)), np.float32(g.uniform(1e-4, 1)), np.float32(g.uniform(0, 50))
        mult = np.float32(np.float32(2) * sg) * dB                              # one rounding
        exact = Fraction(Y) * Fraction(float(mult)) - Fraction(float(nrm))      # then one for the multiply-add
        got = O.score_columns(Y, sg, dB, L2, nrm)
        lo, hi = np.nextafter(got, np.float32(-np.inf)), np.nextafter(got, np.float32(np.inf))
        assert abs(Fraction(float(got)) - exact) <= min(abs(Fraction(float(lo)) - exact), abs(Fraction(float(hi)) - exact))


def test_column_scales_exact_case_equals_brute_force():
    """Factors that the codes represent exactly, with a different power-of-two step size for every column of every
    A_c and for every corpus row: the estimated scores are then the exact inner products <A_c^T q, x_t>, so the search
    without re-ranking must order the points as brute force over rationals does.  A step size taken from the wrong
    column, cluster or row breaks the order."""
    g = np.random.default_rng(13)
    d, L, per = 16, 5, 24
    n = L * per
    f = g.integers(0, 3, size=(L, d))                          # real A_c = diag(2^f_cj)
    f[:, 0] = 2
    e = g.integers(-6, 7, size=n)                              # real row t = 2^e_t * b_t
    b = g.integers(-127, 128, size=(n, d)).astype(np.int64)
    b[:, 1] = 127                                              # every row's absmax code is 127
    A = np.zeros((L, d, d), np.int8)
    A[:, np.arange(d), np.arange(d)] = 64
    ix = dict(metric=IP, n=n, d=d, dp=d, r=d, L=L, centroids=g.normal(size=(L, d)).astype(np.float32), P=None, A=A,
              B=b.astype(np.int8), scale_A=np.ones(L, np.float32), scale_B=np.ones(L, np.float32),
              scale_A_columns=(2.0 ** f / 64).astype(np.float32), scale_B_points=(2.0 ** e).astype(np.float32),
              cluster_offsets=np.arange(L + 1, dtype=np.int64) * per,
              corpus=(b * 2.0 ** e[:, None]).astype(np.float32), ids=None)
    # queries: q_j 2^f_cj / 4 must be an integer for every cluster, and the largest |q_j 2^f_cj| is 127 * 4 (at j = 0)
    Q = (g.integers(-31, 32, size=(12, d)) * 4).astype(np.int64)
    Q[:, 0] = 127
    ids, dists = O.search_no_rerank(O.OracleIndex(ix), Q.astype(np.float32), 9, L)
    for qi in range(len(Q)):
        sc = []
        for t in range(n):
            c = t // per
            sc.append(sum(Fraction(int(Q[qi, j])) * 2 ** int(f[c, j]) * int(b[t, j]) for j in range(d)) * Fraction(2) ** int(e[t]))
        order = sorted(range(n), key=lambda t: (-sc[t], t))[:9]
        assert ids[qi].tolist() == order, qi
        assert [Fraction(float(v)) for v in dists[qi]] == [-sc[t] for t in order]


def test_column_scales_track_float_model_and_beat_cluster_scales(small_indexes, small_indexes_columns):
    """The bound of test_quantized_scores_track_float_model_within_quantization_bound, with the de-quantized factors
    and the half steps of the column-wise scheme; and the reason the paper quantizes column-wise: on the same fitted
    factors the estimated scores are closer to the unquantized model than with one step size per cluster."""
    for name, (wl, ix, corpus, queries) in small_indexes_columns.items():
        a = ix.numpy()
        oix = O.OracleIndex(a)
        _, _, st = O.search(oix, queries, wl.k, wl.w, wl.m, stages=True)
        a1 = small_indexes[name][1].numpy()
        _, _, st1 = O.search(O.OracleIndex(a1), queries, wl.k, wl.w, wl.m, stages=True)
        np.testing.assert_array_equal(st["sel"], st1["sel"])         # routing does not depend on the factors
        err_cols, err_clus = [], []
        for qi in range(0, len(queries), 7):
            for j in range(wl.w):
                c = int(st["sel"][qi, j])
                o0, o1 = int(a["cluster_offsets"][c]), int(a["cluster_offsets"][c + 1])
                if o1 == o0:
                    continue
                dx = float(st["dx"][qi])
                A_real = (a["scale_A_columns"][c].astype(np.float64)[:, None] * a["A"][c].astype(np.float64)).T   # [dp][r]
                B_real = (a["scale_B_points"][o0:o1].astype(np.float64)[:, None] * a["B"][o0:o1].astype(np.float64)).T
                qp = st["qproj"][qi].astype(np.float64)
                y_ref = (qp @ A_real) @ B_real
                sg = float(st["sigma"][qi, j])
                err_r = 0.5 * dx * np.abs(A_real).sum(0) + 0.5 * sg
                bound = err_r @ np.abs(B_real)
                Y = O.pair_accumulators(st["z"][qi, j], a["B"][o0:o1]).astype(np.float64)
                s_hat = sg * a["scale_B_points"][o0:o1].astype(np.float64) * Y
                assert np.all(np.abs(s_hat - y_ref) <= bound * (1 + 1e-4) + 1e-5 * np.abs(y_ref).max()), name
                # both schemes against the UNQUANTIZED fitted model
                y_float = (qp @ a["A_f32"][c].astype(np.float64).T) @ a["B_f32"][o0:o1].astype(np.float64).T
                Y1 = O.pair_accumulators(st1["z"][qi, j], a1["B"][o0:o1]).astype(np.float64)
                err_cols.append(np.abs(s_hat - y_float).mean())
                err_clus.append(np.abs(float(st1["sigma"][qi, j]) * Y1 - y_float).mean())
        assert np.mean(err_cols) < np.mean(err_clus), (name, np.mean(err_cols), np.mean(err_clus))


# ------------------------------------------------------------------ Sec. 4.2: mixed-precision decomposition
def test_mixed_precision_hand_example():
    """The first component of the query and the first rows of A_c and B_c stay in float; only the rest is quantized.
    Numbers chosen so that every float operation is exact."""
    qp = np.array([1000.0, 63.5, -127.0, 0.0, 32.0], np.float32)      # the large first component must not set the step
    q8, dx = O.quantize_query_mixed(qp)
    assert q8.tolist() == [0, 64, -127, 0, 32] and dx == np.float32(1.0)      # 63.5 -> 64 (tie to even)
    A_c = np.array([[99, 2, 0, 0, 0],         # column 0 of A_c (its first entry, 99, must not be read)
                    [-5, 0, 1, 0, 1],         # column 1
                    [7, 1, 1, 0, 0]], np.int8)   # column 2
    dA = np.array([0.5, 0.25, 2.0], np.float32)
    A0 = np.array([0.5, -0.125, 0.0], np.float32)                     # first row of A_c
    R, z, sigma, rho0 = O.stage_a_mixed(q8, float(qp[0]), A_c, float(dx), dA, A0)
    assert R.tolist() == [128, -95, -63]
    # rho = x0 A0 + R dx dA = [500 + 64, -125 - 23.75, 0 - 126] = [564, -148.75, -126]
    assert rho0 == np.float32(564.0)
    assert sigma == np.float32(148.75 / 127)                          # the rest's absmax, not 564
    assert z.tolist() == [0, -127, -108]                              # 126 * 127 / 148.75 = 107.58
    # score: rho0 B0_t on top of the quantized rest, both doubled for Euclidean
    assert O.score_mixed(100, 0.5, 0.25, 564.0, 0.5, IP) == np.float32(12.5 + 282.0)
    assert O.score_mixed(100, 0.5, 0.25, 564.0, 0.5, L2, 3.0) == np.float32(25.0 - 3.0 + 564.0)
    assert O.score_mixed(100, 0.5, 0.25, 0.0, 0.5, COS) == O.score_columns(100, 0.5, 0.25, COS)


def test_mixed_precision_reduces_to_column_scales_without_first_component():
    """A query whose first component is zero, against factors whose first rows are zero, is the column-wise scheme on
    the remaining components: same codes, same step sizes, same results."""
    g = np.random.default_rng(31)
    d, L, per, r = 12, 4, 30, 6
    n = L * per
    A = g.integers(-127, 128, (L, r, d)).astype(np.int8)
    B = g.integers(-127, 128, (n, r)).astype(np.int8)
    A[:, 0, :] = 0; A[:, :, 0] = 0; B[:, 0] = 0       # column 0 of every A_c and the first rows carry nothing
    base = dict(metric=L2, n=n, d=d, dp=d, r=r, L=L, centroids=g.normal(size=(L, d)).astype(np.float32), P=None, A=A, B=B,
                scale_A=np.ones(L, np.float32), scale_B=np.ones(L, np.float32),
                scale_A_columns=g.uniform(0.01, 1, (L, r)).astype(np.float32),
                scale_B_points=g.uniform(0.01, 1, n).astype(np.float32),
                cluster_offsets=np.arange(L + 1, dtype=np.int64) * per,
                corpus=g.normal(size=(n, d)).astype(np.float32), ids=None)
    mixed = dict(base, first_row_A=np.zeros((L, r), np.float32), first_row_B=np.zeros(n, np.float32))
    Q = g.normal(size=(20, d)).astype(np.float32)
    Q[:, 0] = 0.0
    a = O.search(O.OracleIndex(base), Q, 5, 3, 20, stages=True)
    b = O.search(O.OracleIndex(mixed), Q, 5, 3, 20, stages=True)
    for key in ("q8", "dx", "z", "sigma", "cand_rows", "cand_scores"):
        np.testing.assert_array_equal(a[2][key], b[2][key], err_msg=key)
    np.testing.assert_array_equal(a[0], b[0])
    assert not b[2]["rho0"].any()


def test_mixed_precision_exact_case_equals_brute_force():
    """Codes that represent the quantized parts exactly (power-of-two steps) plus small-integer float rows: the
    estimated score is then exactly <q^T A_c, B_c[:, t]> over the full real factors, so the search without
    re-ranking orders the points as brute force over rationals does.  Dropping a float term (x_0 A_c[0][j] for any j,
    r_0 B_c[0][t]), or taking it from the wrong cluster or row, changes the order."""
    g = np.random.default_rng(32)
    d, L, per = 9, 4, 20
    n = L * per
    # real A_c (d x d, r = d): first row a0 in float, below it diag(2^f_cj) on components 1..d-1
    f = g.integers(0, 3, size=(L, d))
    f[:, 1] = 2
    a0 = g.integers(-3, 4, size=(L, d)).astype(np.int64) * 4         # multiples of 4: 127 rho_j / |rho|_inf stays integral
    a0[:, 0] = g.integers(-3, 4, size=L)                              # (r_0 is not quantized: any value)
    a0[:, 1] = 0                                                      # rho_1 = 127 * 4 stays the largest of the rest
    A = np.zeros((L, d, d), np.int8)
    A[:, np.arange(1, d), np.arange(1, d)] = 64
    e = g.integers(-3, 4, size=n)
    b = g.integers(-127, 128, size=(n, d)).astype(np.int64)
    b[:, 0] = 0
    b[:, 2] = 127                                                     # every row's absmax code is 127
    b0 = g.integers(-5, 6, size=n).astype(np.int64)                   # real first row of B_c
    ix = dict(metric=IP, n=n, d=d, dp=d, r=d, L=L, centroids=g.normal(size=(L, d)).astype(np.float32), P=None, A=A,
              B=b.astype(np.int8), scale_A=np.ones(L, np.float32), scale_B=np.ones(L, np.float32),
              scale_A_columns=(2.0 ** f / 64).astype(np.float32), scale_B_points=(2.0 ** e).astype(np.float32),
              first_row_A=a0.astype(np.float32), first_row_B=b0.astype(np.float32),
              cluster_offsets=np.arange(L + 1, dtype=np.int64) * per,
              corpus=g.normal(size=(n, d)).astype(np.float32), ids=None)
    # queries: x_0 a small integer; the rest multiples of 4 with |x_0 a0_j + x_j 2^f_cj| <= 108 + 320 < 508 = rho_1
    Q = (g.integers(-20, 21, size=(10, d)) * 4).astype(np.int64)
    Q[:, 1] = 127
    Q[:, 0] = g.integers(-9, 10, size=10)
    ids, dists = O.search_no_rerank(O.OracleIndex(ix), Q.astype(np.float32), 7, L)
    for qi in range(len(Q)):
        sc = []
        for t in range(n):
            c = t // per
            x0 = int(Q[qi, 0])
            r = [Fraction(x0 * int(a0[c, 0]))] + [Fraction(x0 * int(a0[c, j]) + int(Q[qi, j]) * 2 ** int(f[c, j])) for j in range(1, d)]
            sc.append(r[0] * int(b0[t]) + sum(r[j] * int(b[t, j]) for j in range(1, d)) * Fraction(2) ** int(e[t]))
        order = sorted(range(n), key=lambda t: (-sc[t], t))[:7]
        assert ids[qi].tolist() == order, qi
        assert [Fraction(float(v)) for v in dists[qi]] == [-sc[t] for t in order]


def test_mixed_precision_tracks_float_model_better_when_first_component_dominates(small_indexes_columns, small_indexes_mixed):
    """The reason for the decomposition (Sec. 4.2): after the projection the first component of the query lies on
    the principal axis and dominates the absmax step, so keeping it (and the matching rows) in float leaves finer
    steps for the rest.  On the projected workloads the estimated scores are closer to the unquantized model than
    with the column-wise scheme alone; on every workload they obey the propagated quantization bound."""
    better = []
    for name, (wl, ix, corpus, queries) in small_indexes_mixed.items():
        a = ix.numpy()
        _, _, st = O.search(O.OracleIndex(a), queries, wl.k, wl.w, wl.m, stages=True)
        ac = small_indexes_columns[name][1].numpy()
        _, _, sc = O.search(O.OracleIndex(ac), queries, wl.k, wl.w, wl.m, stages=True)
        err_mixed, err_cols = [], []
        for qi in range(0, len(queries), 7):
            qp = st["qproj"][qi].astype(np.float64)
            for j in range(wl.w):
                c = int(st["sel"][qi, j])
                o0, o1 = int(a["cluster_offsets"][c]), int(a["cluster_offsets"][c + 1])
                if o1 == o0:
                    continue
                y_float = (qp @ a["A_f32"][c].astype(np.float64).T) @ a["B_f32"][o0:o1].astype(np.float64).T
                sg, r0 = float(st["sigma"][qi, j]), float(st["rho0"][qi, j])
                Y = O.pair_accumulators(st["z"][qi, j], a["B"][o0:o1]).astype(np.float64)
                s_hat = r0 * a["first_row_B"][o0:o1].astype(np.float64) + sg * a["scale_B_points"][o0:o1].astype(np.float64) * Y
                # bound: half a step per quantized query component through |A|, half a step of z through |B|
                A_real = (a["scale_A_columns"][c].astype(np.float64)[:, None] * a["A"][c].astype(np.float64)).T   # [dp][r], row 0 zero
                B_real = (a["scale_B_points"][o0:o1].astype(np.float64)[:, None] * a["B"][o0:o1].astype(np.float64)).T
                y_ref = (qp[1:] @ A_real[1:] + qp[0] * a["first_row_A"][c].astype(np.float64))
                y_ref = y_ref[0] * a["first_row_B"][o0:o1].astype(np.float64) + y_ref[1:] @ B_real[1:]
                err_r = 0.5 * float(st["dx"][qi]) * np.abs(A_real[1:]).sum(0) + 0.5 * sg
                err_r[0] = 0.5 * float(st["dx"][qi]) * np.abs(A_real[1:, 0]).sum()
                bound = err_r[1:] @ np.abs(B_real[1:]) + err_r[0] * np.abs(a["first_row_B"][o0:o1].astype(np.float64))
                assert np.all(np.abs(s_hat - y_ref) <= bound * (1 + 1e-4) + 1e-5 * np.abs(y_ref).max()), name
                if wl.dp < wl.d and int(sc["sel"][qi, j]) == c:
                    # (the two builds rotate differently, so each is compared with its own unquantized model)
                    qpc = sc["qproj"][qi].astype(np.float64)
                    y_float_c = (qpc @ ac["A_f32"][c].astype(np.float64).T) @ ac["B_f32"][o0:o1].astype(np.float64).T
                    Yc = O.pair_accumulators(sc["z"][qi, j], ac["B"][o0:o1]).astype(np.float64)
                    s_c = float(sc["sigma"][qi, j]) * ac["scale_B_points"][o0:o1].astype(np.float64) * Yc
                    err_mixed.append(np.abs(s_hat - y_float).mean() / (np.abs(y_float).mean() + 1e-30))
                    err_cols.append(np.abs(s_c - y_float_c).mean() / (np.abs(y_float_c).mean() + 1e-30))
        if err_mixed:
            better.append((name, float(np.mean(err_mixed)), float(np.mean(err_cols))))
    assert better, "no projected workload among the small ones"
    print(better)
    assert all(m < c for _, m, c in better), better


# ------------------------------------------------------------------ Sec. 2.2 / 3.1 / 4.1: routing, selection, re-rank
def test_projection_is_matrix_product():
    """Sec. 4.1: x' = W_s^T x."""
    q = rng.normal(size=37).astype(np.float32)
    P = rng.normal(size=(37, 11)).astype(np.float32)
    np.testing.assert_array_equal(O.project(q, P), (q.astype(np.float64) @ P.astype(np.float64)).astype(np.float32))
    np.testing.assert_array_equal(O.project(q, None), q)


def test_centroid_dissimilarities_and_routing_order():
    """Sec. 2.2 (w nearest centroids), Sec. 3.1 (Euclidean ranking through -2 x^T c + |c|^2): the routing
    order equals the order of true squared distances / negative inner products; ties go to the lower id."""
    dp, L = 20, 50
    cent = rng.normal(size=(L, dp)).astype(np.float32)
    cent[17] = cent[3]                                        # exact tie between clusters 3 and 17
    qp = rng.normal(size=dp).astype(np.float32)
    c64, q64 = cent.astype(np.float64), qp.astype(np.float64)
    g_ip = O.centroid_dissim(qp, cent, IP)
    np.testing.assert_allclose(g_ip, -(c64 @ q64), rtol=1e-6)
    np.testing.assert_array_equal(O.centroid_dissim(qp, cent, COS), g_ip)
    g_l2 = O.centroid_dissim(qp, cent, L2)
    d2 = ((c64 - q64) ** 2).sum(1)
    np.testing.assert_allclose(g_l2 + (q64 @ q64), d2, rtol=1e-5, atol=1e-5)
    for g in (g_ip, g_l2):
        sel, sg = O.select_clusters(g, 12)
        order = np.lexsort((np.arange(L), g))[:12]
        np.testing.assert_array_equal(sel, order)
        np.testing.assert_array_equal(sg, g[order])
    sel, _ = O.select_clusters(g_l2, L)
    assert list(sel).index(3) + 1 == list(sel).index(17)       # tie: lower id first


def test_dissimilarity_identities():
    """Sec. 2.1 + 3.1: |q - c|^2 = |q|^2 + |c|^2 - 2<q,c>; cosine distance equals 1 - <q,c>/|q| for a
    unit-norm corpus point and is scale-invariant in q."""
    for _ in range(20):
        d = int(rng.integers(1, 200))
        q = rng.normal(size=d).astype(np.float32)
        c = rng.normal(size=d).astype(np.float32)
        l2, ip = float(O.exact_dissim(q, c, L2)), float(O.exact_dissim(q, c, IP))
        qn, cn = float(O.row_sqnorm(q)), float(O.row_sqnorm(c))
        assert l2 == pytest.approx(qn + cn + 2 * ip, rel=1e-5, abs=1e-5)
        cu = (c / np.linalg.norm(c)).astype(np.float32)
        cos = float(O.exact_dissim(q, cu, COS))
        ref = 1 - float(q.astype(np.float64) @ cu.astype(np.float64)) / np.linalg.norm(q.astype(np.float64))
        assert cos == pytest.approx(ref, abs=1e-6)
        assert float(O.exact_dissim((3 * q).astype(np.float32), cu, COS)) == pytest.approx(cos, abs=1e-6)
    assert O.exact_dissim(np.zeros(4, np.float32), np.ones(4, np.float32), COS) == 1.0


def test_score_is_one_fused_multiply_add():
    """Sec. 3.1: Euclidean candidates are ranked by 2 x^T c - |c|^2 (negated argmin form); inner product and
    cosine by the estimate itself."""
    assert O.score(1000, 0.5, IP) == 500.0
    assert O.score(-7, 0.25, COS) == -1.75
    assert O.score(1000, 0.5, L2, 10.0) == 990.0
    # single rounding: 2*sigma*Y - n differs from the twice-rounded product-then-subtract
    Y, s, nrm = 12345, np.float32(0.1), np.float32(2468.9)
    exact = float(np.float32(Y)) * float(np.float32(2) * s) - float(nrm)
    assert O.score(Y, s, L2, nrm) == np.float32(exact)


def _numpy_knn(corpus, q, metric, k, ids):
    c, x = corpus.astype(np.float64), q.astype(np.float64)
    if metric == L2:
        dis = ((c - x) ** 2).sum(1)
    elif metric == IP:
        dis = -(c @ x)
    else:
        dis = 1 - (c @ x) / np.linalg.norm(x)
    dis32 = dis.astype(np.float32)
    order = np.lexsort((ids, dis32))[:k]
    return ids[order], dis32[order]


def test_probing_everything_returns_exact_knn(small_indexes):
    """Sec. 2.1 Eq. (1) + Sec. 2.2: with every cluster probed and every point kept as candidate the
    pipeline reduces to exact k-NN, whatever the quality of the 8-bit scores: brute force in numpy."""
    for name, (wl, ix, corpus, queries) in small_indexes.items():
        a = ix.numpy()
        oix = O.OracleIndex(a)
        ids, dists = O.search(oix, queries[:15], wl.k, wl.L, wl.n)
        for qi in range(15):
            e_ids, e_d = _numpy_knn(a["corpus"], queries[qi], wl.metric, wl.k, a["ids"])
            np.testing.assert_allclose(dists[qi], e_d, rtol=1e-5, atol=1e-6, err_msg=name)
            assert np.array_equal(ids[qi], e_ids) or np.allclose(dists[qi], e_d, rtol=1e-6), name
        # the oracle's own exhaustive k-NN (used for recall) agrees as well
        k_ids, k_d = O.exact_knn(a["corpus"], queries[:15], wl.metric, wl.k, ids=a["ids"])
        np.testing.assert_array_equal(k_ids, ids)
        np.testing.assert_array_equal(k_d, dists)


def test_returned_ids_refer_to_original_corpus(small_indexes):
    """Rows are stored in cluster order; returned ids are original corpus indices."""
    wl, ix, corpus, queries = small_indexes["ip_P"]
    a = ix.numpy()
    np.testing.assert_array_equal(corpus[a["ids"]], a["corpus"])
    ids, dists = O.search(O.OracleIndex(a), queries[:5], wl.k, wl.w, wl.m)
    for qi in range(5):
        for t in range(wl.k):
            ref = -float(corpus[ids[qi, t]].astype(np.float64) @ queries[qi].astype(np.float64))
            assert dists[qi, t] == pytest.approx(ref, rel=1e-6, abs=1e-7)


def test_candidate_set_and_rerank_follow_the_template(small_indexes):
    """Sec. 2.2: score the points of the w selected clusters, keep the m best, re-rank them with the true
    dissimilarity of the ORIGINAL query (Sec. 4.1), return the k best.  Recomputed here step by step in
    numpy from the stage outputs."""
    for name, (wl, ix, corpus, queries) in small_indexes.items():
        a = ix.numpy()
        oix = O.OracleIndex(a)
        ids, dists, st = O.search(oix, queries, wl.k, wl.w, wl.m, stages=True)
        off = a["cluster_offsets"]
        for qi in range(0, len(queries), 5):
            rows, scores = [], []
            for j in range(wl.w):
                c = int(st["sel"][qi, j])
                o0, o1 = int(off[c]), int(off[c + 1])
                Y = a["B"][o0:o1].astype(np.int64) @ st["z"][qi, j].astype(np.int64)
                sg = np.float32(st["sigma"][qi, j])
                if wl.metric == L2:
                    nrm = (a["corpus"][o0:o1].astype(np.float64) ** 2).sum(1).astype(np.float32)
                    s = (Y.astype(np.float64) * float(np.float32(2) * sg) - nrm.astype(np.float64)).astype(np.float32)
                else:
                    s = (Y.astype(np.float64) * float(sg)).astype(np.float32)
                rows.append(np.arange(o0, o1))
                scores.append(s)
                # the exported best score of the pair is the largest of these (-inf for an empty cluster)
                assert st["pair_best"][qi, j] == (s.max() if s.size else -np.inf), name
            rows, scores = np.concatenate(rows), np.concatenate(scores)
            assert st["cand_scores"][qi, 0] == st["pair_best"][qi].max()
            order = np.lexsort((rows, -scores.astype(np.float64)))[:wl.m]
            nc = len(order)
            np.testing.assert_array_equal(st["cand_rows"][qi, :nc], rows[order], err_msg=name)
            assert np.all(st["cand_rows"][qi, nc:] == -1)
            np.testing.assert_array_equal(st["cand_scores"][qi, :nc], scores[order])
            e_ids, e_d = _numpy_knn(a["corpus"][rows[order]], queries[qi], wl.metric, wl.k, a["ids"][rows[order]])
            np.testing.assert_array_equal(ids[qi, :len(e_ids)], e_ids)
            np.testing.assert_allclose(dists[qi, :len(e_ids)], e_d, rtol=1e-6, atol=1e-7)


def test_no_rerank_variant_returns_the_best_estimated_scores(small_indexes):
    """Sec. 7.1 (memory usage) / App. D.3: without the final re-ranking step the answer is the k points of highest
    estimated score.  Recomputed in numpy from the stage outputs (integer products, one rounding per score)."""
    for name, (wl, ix, corpus, queries) in small_indexes.items():
        a = ix.numpy()
        oix = O.OracleIndex(a)
        _, _, st = O.search(oix, queries, wl.k, wl.w, wl.m, stages=True)
        ids, dists = O.search_no_rerank(oix, queries, wl.k, wl.w)
        off = a["cluster_offsets"]
        for qi in range(0, len(queries), 3):
            rows, scores = [], []
            for j in range(wl.w):
                c = int(st["sel"][qi, j])
                o0, o1 = int(off[c]), int(off[c + 1])
                Y = a["B"][o0:o1].astype(np.int64) @ st["z"][qi, j].astype(np.int64)
                sg = np.float32(st["sigma"][qi, j])
                if wl.metric == L2:
                    nrm = (a["corpus"][o0:o1].astype(np.float64) ** 2).sum(1).astype(np.float32)
                    s = (Y.astype(np.float64) * float(np.float32(2) * sg) - nrm.astype(np.float64)).astype(np.float32)
                else:
                    s = (Y.astype(np.float64) * float(sg)).astype(np.float32)
                rows.append(np.arange(o0, o1))
                scores.append(s)
            rows, scores = np.concatenate(rows), np.concatenate(scores)
            best = np.lexsort((rows, -scores.astype(np.float64)))[:wl.k]       # boundary ties: lower row
            e_ids, e_d = a["ids"][rows[best]], -scores[best]
            order = np.lexsort((e_ids, e_d))                                     # reported order: (dissimilarity, id)
            np.testing.assert_array_equal(ids[qi], e_ids[order], err_msg=name)
            np.testing.assert_array_equal(dists[qi], e_d[order], err_msg=name)


def test_no_rerank_variant_with_exact_factors_is_exact_search():
    """With integer data that the 8-bit codes represent exactly (A_c = 127 I, rows and queries integer vectors whose
    largest entry is 127) every estimated score is a known multiple of the true inner product, so the variant without
    re-ranking must return the exact nearest neighbours by inner product: brute force with Python integers."""
    g = np.random.default_rng(5)
    d, L, per = 16, 4, 30
    n = L * per
    rows = g.integers(-127, 128, size=(n, d)).astype(np.int64)
    A = np.zeros((L, d, d), np.int8)
    A[:, np.arange(d), np.arange(d)] = 127
    ix = dict(metric=IP, n=n, d=d, dp=d, r=d, L=L, centroids=g.normal(size=(L, d)).astype(np.float32), P=None, A=A,
              B=rows.astype(np.int8), scale_A=np.full(L, 1 / 127, np.float32), scale_B=np.ones(L, np.float32),
              cluster_offsets=np.arange(L + 1, dtype=np.int64) * per, corpus=rows.astype(np.float32), ids=None)
    Q = g.integers(-126, 127, size=(20, d)).astype(np.int64)
    Q[:, 0] = 127                                  # absmax 127: the query codes are the query itself
    ids, dists = O.search_no_rerank(O.OracleIndex(ix), Q.astype(np.float32), 7, L)
    for qi in range(len(Q)):
        ip = [int(sum(int(a) * int(b) for a, b in zip(rows[j], Q[qi]))) for j in range(n)]
        # every R_j equals 127 q_j, so max|R| = 127 * 127, z = q and sigma = 1: the score is the inner product itself
        order = sorted(range(n), key=lambda j: (-ip[j], j))[:7]
        assert ids[qi].tolist() == order, qi
        np.testing.assert_allclose(dists[qi], [-ip[j] for j in order], rtol=2e-7)


def test_half_precision_rerank_rows():
    """Sec. 4.3 (16-bit floating point on the GPU): the re-rank over a binary16 copy of the corpus is the plain
    re-rank over the rounded rows.  Pins of the rounding (nearest, ties to even, gradual underflow) on hand-computed
    values, and of the search against brute force over the rounded rows."""
    x = np.array([1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11, 1 + 2.0 ** -11 + 2.0 ** -20, 65504.0, 2.0 ** -24, 2.0 ** -25,
                  3 * 2.0 ** -25, -0.1], np.float32)
    want = np.array([1.0, 1 + 2.0 ** -9, 1 + 2.0 ** -10, 65504.0, 2.0 ** -24, 0.0, 2.0 ** -23, -0.0999755859375],
                    np.float32)
    got = O.with_half_precision_corpus(dict(corpus=x.reshape(1, -1)))["rerank_corpus"].ravel()
    np.testing.assert_array_equal(got, want)


def test_half_precision_rerank_search(small_indexes):
    for name, (wl, ix, corpus, queries) in small_indexes.items():
        a = O.with_half_precision_corpus(ix.numpy())
        rounded = a["rerank_corpus"]
        assert np.abs(rounded - a["corpus"]).max() <= 2.0 ** -11 * np.abs(a["corpus"]).max()
        oix = O.OracleIndex(a)
        ids, dists = O.search(oix, queries[:15], wl.k, wl.L, wl.n)          # everything probed and kept: exact k-NN
        for qi in range(15):
            e_ids, e_d = _numpy_knn(rounded, queries[qi], wl.metric, wl.k, a["ids"])
            np.testing.assert_allclose(dists[qi], e_d, rtol=1e-5, atol=1e-6, err_msg=name)
            assert np.array_equal(ids[qi], e_ids) or np.allclose(dists[qi], e_d, rtol=1e-6), name
        # the candidate sets do not depend on the re-rank rows (the Euclidean score keeps the original norms)
        _, _, st_h = O.search(oix, queries, wl.k, wl.w, wl.m, stages=True)
        _, _, st_f = O.search(O.OracleIndex(ix.numpy()), queries, wl.k, wl.w, wl.m, stages=True)
        np.testing.assert_array_equal(st_h["cand_rows"], st_f["cand_rows"])
        np.testing.assert_array_equal(st_h["cand_scores"], st_f["cand_scores"])


def test_fewer_candidates_than_k_pads():
    """Fewer scored points than k: remaining slots hold id -1 and distance +inf."""
    d, L = 8, 3
    corpus = rng.normal(size=(4, d)).astype(np.float32)
    ix = dict(metric=IP, n=4, d=d, dp=d, r=8, L=L, centroids=rng.normal(size=(L, d)).astype(np.float32), P=None,
              A=rng.integers(-127, 128, size=(L, 8, d)).astype(np.int8),
              B=rng.integers(-127, 128, size=(4, 8)).astype(np.int8), scale_A=np.ones(L, np.float32),
              scale_B=np.ones(L, np.float32), cluster_offsets=np.array([0, 2, 2, 4], np.int64), corpus=corpus, ids=None)
    q = corpus[:1] * 2
    ids, dists = O.search(O.OracleIndex(ix), q, 6, 3, 10)
    assert sorted(ids[0, :4].tolist()) == [0, 1, 2, 3] and ids[0, 4:].tolist() == [-1, -1]
    assert np.isinf(dists[0, 4:]).all() and np.all(np.diff(dists[0, :4]) >= 0)
    with pytest.raises(ValueError):
        O.search(O.OracleIndex(ix), q, 6, 4, 10)          # w > L
    with pytest.raises(ValueError):
        O.search(O.OracleIndex(ix), q, 6, 2, 5)           # k > m


# ------------------------------------------------------------------ Sec. 3.3 / 4.2: memory
def test_index_bytes_match_memory_model(small_indexes):
    """Sec. 4.2: the factors take L*s*r + r*m bytes."""
    for name, (wl, ix, _, _) in small_indexes.items():
        a = ix.numpy()
        assert a["A"].nbytes + a["B"].nbytes == wl.L * wl.dp * wl.r + wl.r * wl.n
        assert a["A"].dtype == np.int8 and a["B"].dtype == np.int8
