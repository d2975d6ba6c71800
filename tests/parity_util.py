"""Comparison helpers shared by the GPU parity tests."""
import numpy as np

from oracle import oracle as O

DIST_RTOL = 1e-4      # float re-rank distances: GPU accumulates in fp32, the oracle in fp64
TIE_RTOL = 1e-5       # returned ids may differ only where the distances tie within this relative tolerance
TIE_FLOOR = 1e-3      # ... measured against max(|distance|, TIE_FLOOR)


def rounding_abs_tol(queries, corpus, metric):
    """Absolute error bound of an inner product accumulated in fp32: d * 2^-24 * |q| * max|x| per query (for the
    cosine dissimilarity the product is divided by |q|).  Only inner-product-like results can cancel to values far
    below the size of their terms; for them DIST_RTOL relative to the result itself says nothing about the
    arithmetic, and this bound is added to it.  Euclidean distances are sums of squares and need no such term."""
    queries, corpus = np.asarray(queries, np.float64), np.asarray(corpus, np.float64)
    d = queries.shape[1]
    xmax = float(np.sqrt((corpus * corpus).sum(axis=1).max()))
    qn = np.sqrt((queries * queries).sum(axis=1))
    if metric == 1:
        return np.full(queries.shape[0], 1e-7)
    if metric == 2:
        return np.full(queries.shape[0], d * 2.0 ** -24 * xmax + 1e-7)
    return d * 2.0 ** -24 * qn * xmax + 1e-7


def oracle_distance_of(index_arrays, queries, rerank_corpus=None):
    """(query number, returned id) -> the oracle's exact dissimilarity of that point (step 7 of the oracle), for
    judging a returned id that the oracle's own list does not contain."""
    corpus = np.asarray(index_arrays["corpus"] if rerank_corpus is None else rerank_corpus, np.float32)
    ids = index_arrays.get("ids")
    metric = int(index_arrays["metric"])
    row_of = {}

    def f(qi, pid):
        if ids is not None and not row_of:        # built on first use: most comparisons never ask
            inv = np.argsort(np.asarray(ids), kind="stable")
            row_of["sorted"], row_of["rows"] = np.asarray(ids)[inv], inv
        row = int(pid) if ids is None else int(row_of["rows"][np.searchsorted(row_of["sorted"], int(pid))])
        return float(O.exact_dissim(queries[qi], corpus[row], metric))
    return f


def assert_topk_equal(ids_gpu, dists_gpu, ids_ref, dists_ref, what="", abs_tol=1e-7, exact=None):
    """Distances within DIST_RTOL relative (plus `abs_tol`, scalar or one value per query: see rounding_abs_tol);
    ids identical except at ties: a differing id is accepted only if it is another member of the oracle's list at
    a tied distance, or - when the oracle's list does not hold it - if the oracle's own distance of that point
    (`exact`, see oracle_distance_of) ties with the last distance of the oracle's list and so does the entry it
    displaced.  Returns the number of differing positions."""
    ids_gpu, ids_ref = np.asarray(ids_gpu), np.asarray(ids_ref)
    dists_gpu, dists_ref = np.asarray(dists_gpu, np.float64), np.asarray(dists_ref, np.float64)
    assert ids_gpu.shape == ids_ref.shape and dists_gpu.shape == dists_ref.shape, what
    pad = ids_ref < 0
    assert np.array_equal(pad, ids_gpu < 0), f"{what}: padding differs"
    assert np.all(np.isinf(dists_gpu[pad])), what
    ok = ~pad
    tol = DIST_RTOL * np.abs(dists_ref) + np.broadcast_to(np.asarray(abs_tol, np.float64).reshape(-1, 1) if np.ndim(abs_tol) else abs_tol, dists_ref.shape)
    err = np.abs(np.where(ok, dists_gpu, 0.0) - np.where(ok, dists_ref, 0.0))
    bad = ok & ~(err <= tol)
    assert not bad.any(), f"{what}: distance error {err[bad].max():.3g} (allowed {tol[bad].min():.3g}) at {np.argwhere(bad)[0]}"
    mism = ok & (ids_gpu != ids_ref)
    for qi in np.unique(np.nonzero(mism)[0]):
        dr = dists_ref[qi]
        last = int(np.nonzero(ok[qi])[0].max())
        for c in np.nonzero(mism[qi])[0]:
            win = TIE_RTOL * max(abs(dr[c]), TIE_FLOOR)
            g = ids_gpu[qi, c]
            where = np.nonzero(ok[qi] & (ids_ref[qi] == g))[0]
            if where.size:
                tied = abs(dr[where[0]] - dr[c]) <= win
                assert tied, f"{what}: query {qi} position {c}: id {g} vs {ids_ref[qi, c]} is not a tie"
            else:
                # the point is not in the oracle's list: it can only have displaced entries that tie with the list's end
                assert exact is not None, f"{what}: query {qi} position {c}: id {g} is not in the oracle's list"
                dg = exact(qi, g)
                tied = abs(dg - dr[last]) <= TIE_RTOL * max(abs(dr[last]), TIE_FLOOR) and abs(dr[c] - dr[last]) <= win
                assert tied, f"{what}: query {qi} position {c}: id {g} (oracle distance {dg}) does not tie with the list's end {dr[last]}"
    return int(mism.sum())


def y_offsets(sel, cluster_offsets):
    """Offsets of every (query, rank) slot into the flat integer-score dump."""
    sizes = (cluster_offsets[1:] - cluster_offsets[:-1])[sel.reshape(-1)]
    off = np.zeros(sizes.size + 1, np.int64)
    np.cumsum(sizes, out=off[1:])
    return off
