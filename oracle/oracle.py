"""ctypes front end of the C oracle (oracle/lorann_oracle.c).  TEST INFRASTRUCTURE ONLY.

Every function takes and returns numpy arrays on the host.  The index is a dict with the keys of the
library's load call: metric, n, d, dp, r, L, centroids, P (or None), A, B, scale_A, scale_B,
cluster_offsets, corpus, ids (or None).
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


class _Index(C.Structure):
    _fields_ = [("metric", C.c_int32), ("n", C.c_int64), ("d", C.c_int32), ("dp", C.c_int32), ("r", C.c_int32),
                ("L", C.c_int32), ("centroids", C.c_void_p), ("P", C.c_void_p), ("A", C.c_void_p),
                ("B", C.c_void_p), ("scale_A", C.c_void_p), ("scale_B", C.c_void_p), ("offsets", C.c_void_p),
                ("corpus", C.c_void_p), ("ids", C.c_void_p), ("sqnorms", C.c_void_p),
                ("col_scale_A", C.c_void_p), ("pt_scale_B", C.c_void_p),
                ("first_row_A", C.c_void_p), ("first_row_B", C.c_void_p)]


class _Dump(C.Structure):
    _fields_ = [(name, C.c_void_p) for name in
                ("qproj", "q8", "dx", "sel", "sel_g", "R", "z", "sigma", "cand_rows", "cand_scores", "rho0", "pair_best")]


def lib():
    global _lib
    if _lib is None:
        path = os.environ.get("LORANN_ORACLE_LIB") or _build.build(force=False)   # (the sanitized build, for the test that runs the pins under it)
        _lib = C.CDLL(str(path))
        _lib.oracle_search.restype = C.c_int
        _lib.oracle_exact_knn.restype = C.c_int
        _lib.oracle_search_no_rerank.restype = C.c_int
        _lib.oracle_row_sqnorm.restype = C.c_float
        _lib.oracle_score.restype = C.c_float
        _lib.oracle_score.argtypes = [C.c_int32, C.c_float, C.c_int32, C.c_float]
        _lib.oracle_exact_dissim.restype = C.c_float
        _lib.oracle_score_columns.restype = C.c_float
        _lib.oracle_score_columns.argtypes = [C.c_int32, C.c_float, C.c_float, C.c_int32, C.c_float]
        _lib.oracle_score_mixed.restype = C.c_float
        _lib.oracle_score_mixed.argtypes = [C.c_int32, C.c_float, C.c_float, C.c_float, C.c_float, C.c_int32, C.c_float]
        _lib.oracle_load_file.restype = C.POINTER(_Index)
        _lib.oracle_load_file.argtypes = [C.c_char_p]
        _lib.oracle_free_loaded.restype = None
        _lib.oracle_free_loaded.argtypes = [C.POINTER(_Index)]
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a, dtype):
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


class OracleIndex:
    """Host-side view of an index for the oracle (keeps the arrays alive; precomputes |c_j|^2 for L2)."""

    def __init__(self, ix: dict):
        self.metric, self.n, self.d, self.dp, self.r, self.L = (int(ix[k]) for k in ("metric", "n", "d", "dp", "r", "L"))
        self.centroids = _c(ix["centroids"], np.float32)
        self.P = _c(ix.get("P"), np.float32)
        self.A = _c(ix["A"], np.int8)
        self.B = _c(ix["B"], np.int8)
        self.scale_A = _c(ix["scale_A"], np.float32)
        self.scale_B = _c(ix["scale_B"], np.float32)
        self.offsets = _c(ix["cluster_offsets"], np.int64)
        self.corpus = _c(ix["corpus"], np.float32)
        self.ids = _c(ix.get("ids"), np.int64)
        assert self.centroids.shape == (self.L, self.dp) and self.A.shape == (self.L, self.r, self.dp)
        assert self.B.shape == (self.n, self.r) and self.corpus.shape == (self.n, self.d)
        assert self.offsets.shape == (self.L + 1,) and self.offsets[0] == 0 and self.offsets[-1] == self.n
        assert self.P is None or self.P.shape == (self.d, self.dp)
        self.sqnorms = None
        if self.metric == 1:
            self.sqnorms = np.empty(self.n, np.float32)
            lib().oracle_corpus_sqnorms(_p(self.corpus), C.c_int64(self.n), C.c_int32(self.d), _p(self.sqnorms))
        # optional: the rows the re-rank reads, when they are not the corpus the index was built from
        self.rerank_corpus = _c(ix.get("rerank_corpus"), np.float32)
        assert self.rerank_corpus is None or self.rerank_corpus.shape == self.corpus.shape
        # optional: one step size per column of A_c and of B_c (Sec. 3.3 as printed) instead of one per cluster
        self.scale_A_columns = _c(ix.get("scale_A_columns"), np.float32)
        self.scale_B_points = _c(ix.get("scale_B_points"), np.float32)
        assert (self.scale_A_columns is None) == (self.scale_B_points is None)
        if self.scale_A_columns is not None:
            assert self.scale_A_columns.shape == (self.L, self.r) and self.scale_B_points.shape == (self.n,)
        # optional (with the column step sizes): unquantized first rows of A_c and B_c (Sec. 4.2 mixed precision)
        self.first_row_A = _c(ix.get("first_row_A"), np.float32)
        self.first_row_B = _c(ix.get("first_row_B"), np.float32)
        assert (self.first_row_A is None) == (self.first_row_B is None)
        if self.first_row_A is not None:
            assert self.scale_A_columns is not None
            assert self.first_row_A.shape == (self.L, self.r) and self.first_row_B.shape == (self.n,)
        self.c = _Index(self.metric, self.n, self.d, self.dp, self.r, self.L, _p(self.centroids), _p(self.P),
                        _p(self.A), _p(self.B), _p(self.scale_A), _p(self.scale_B), _p(self.offsets),
                        _p(self.corpus if self.rerank_corpus is None else self.rerank_corpus), _p(self.ids),
                        _p(self.sqnorms), _p(self.scale_A_columns), _p(self.scale_B_points), _p(self.first_row_A),
                        _p(self.first_row_B))


def _from_file(path) -> "OracleIndex":
    """The oracle's own reader of the serialized index file (the C routine parses it; numpy only views its arrays)."""
    p = lib().oracle_load_file(str(path).encode())
    if not p:
        raise ValueError(f"oracle: cannot load index file {path}")
    c = p.contents
    self = OracleIndex.__new__(OracleIndex)
    self._loaded = p
    self.metric, self.n, self.d, self.dp, self.r, self.L = c.metric, c.n, c.d, c.dp, c.r, c.L

    def view(ptr, ctype, shape):
        if not ptr:
            return None
        return np.ctypeslib.as_array(C.cast(ptr, C.POINTER(ctype)), shape=shape)

    self.centroids = view(c.centroids, C.c_float, (c.L, c.dp))
    self.P = view(c.P, C.c_float, (c.d, c.dp))
    self.A = view(c.A, C.c_int8, (c.L, c.r, c.dp))
    self.B = view(c.B, C.c_int8, (c.n, c.r))
    self.scale_A = view(c.scale_A, C.c_float, (c.L,))
    self.scale_B = view(c.scale_B, C.c_float, (c.L,))
    self.offsets = view(c.offsets, C.c_int64, (c.L + 1,))
    self.corpus = view(c.corpus, C.c_float, (c.n, c.d))
    self.ids = view(c.ids, C.c_int64, (c.n,))
    self.sqnorms = view(c.sqnorms, C.c_float, (c.n,))
    self.c = c
    return self


def _release(self):
    p = getattr(self, "_loaded", None)
    if p:
        self._loaded = None
        lib().oracle_free_loaded(p)


OracleIndex.from_file = staticmethod(_from_file)
OracleIndex.__del__ = _release


def default_threads() -> int:
    return len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)


def search(oix: OracleIndex, Q, k: int, w: int, m: int, stages: bool = False, threads: int | None = None):
    """Run the query phase.  Returns (ids [nq,k] int64, dists [nq,k] f32) and, with stages=True, a dict of
    the intermediate arrays of every step."""
    Q = _c(Q, np.float32)
    nq = Q.shape[0]
    assert Q.ndim == 2 and Q.shape[1] == oix.d
    ids = np.empty((nq, k), np.int64)
    dists = np.empty((nq, k), np.float32)
    st, dump = None, None
    if stages:
        st = dict(qproj=np.zeros((nq, oix.dp), np.float32), q8=np.zeros((nq, oix.dp), np.int8),
                  dx=np.zeros(nq, np.float32), sel=np.zeros((nq, w), np.int32), sel_g=np.zeros((nq, w), np.float32),
                  R=np.zeros((nq, w, oix.r), np.int32), z=np.zeros((nq, w, oix.r), np.int8),
                  sigma=np.zeros((nq, w), np.float32), cand_rows=np.zeros((nq, m), np.int64),
                  cand_scores=np.zeros((nq, m), np.float32), rho0=np.zeros((nq, w), np.float32),
                  pair_best=np.zeros((nq, w), np.float32))
        dump = _Dump(*[_p(st[f[0]]) for f in _Dump._fields_])
    rc = lib().oracle_search(C.byref(oix.c), _p(Q), C.c_int64(nq), C.c_int32(k), C.c_int32(w), C.c_int32(m),
                             _p(ids), _p(dists), C.byref(dump) if dump is not None else None,
                             C.c_int32(threads or default_threads()))
    if rc != 0:
        raise ValueError("oracle_search: invalid arguments")
    return (ids, dists, st) if stages else (ids, dists)


def search_no_rerank(oix: OracleIndex, Q, k: int, w: int, threads: int | None = None):
    """The query phase without the final re-ranking step: the k highest estimated scores, dists = -score."""
    Q = _c(Q, np.float32)
    nq = Q.shape[0]
    assert Q.ndim == 2 and Q.shape[1] == oix.d
    ids = np.empty((nq, k), np.int64)
    dists = np.empty((nq, k), np.float32)
    rc = lib().oracle_search_no_rerank(C.byref(oix.c), _p(Q), C.c_int64(nq), C.c_int32(k), C.c_int32(w), _p(ids),
                                       _p(dists), C.c_int32(threads or default_threads()))
    if rc != 0:
        raise ValueError("oracle_search_no_rerank: invalid arguments")
    return ids, dists


def with_half_precision_corpus(ix: dict) -> dict:
    """The index whose re-rank reads a 16-bit floating-point copy of the corpus (Sec. 4.3: 16-bit floating point
    on the GPU): every corpus value rounded to IEEE binary16 (numpy's conversion: round to nearest, ties to even)
    and widened back exactly.  Everything else is unchanged; in particular the row norms inside the Euclidean
    score (Sec. 3.1) stay those of the original rows, they belong to the index."""
    out = dict(ix)
    out["rerank_corpus"] = np.asarray(ix["corpus"], np.float32).astype(np.float16).astype(np.float32)
    return out


def exact_knn(corpus, Q, metric: int, k: int, ids=None, threads: int | None = None):
    corpus, Q, ids = _c(corpus, np.float32), _c(Q, np.float32), _c(ids, np.int64)
    nq, n, d = Q.shape[0], corpus.shape[0], corpus.shape[1]
    out_i = np.empty((nq, k), np.int64)
    out_d = np.empty((nq, k), np.float32)
    rc = lib().oracle_exact_knn(_p(corpus), C.c_int64(n), C.c_int32(d), C.c_int32(metric), _p(ids), _p(Q),
                                C.c_int64(nq), C.c_int32(k), _p(out_i), _p(out_d),
                                C.c_int32(threads or default_threads()))
    if rc != 0:
        raise ValueError("oracle_exact_knn: invalid arguments")
    return out_i, out_d


def project(q, P):
    q = _c(q, np.float32)
    P = _c(P, np.float32)
    d = q.shape[0]
    dp = d if P is None else P.shape[1]
    out = np.empty(dp, np.float32)
    lib().oracle_project(_p(q), C.c_int32(d), C.c_int32(dp), _p(P), _p(out))
    return out


def centroid_dissim(qp, centroids, metric: int):
    qp, centroids = _c(qp, np.float32), _c(centroids, np.float32)
    g = np.empty(centroids.shape[0], np.float32)
    lib().oracle_centroid_dissim(_p(qp), C.c_int32(qp.shape[0]), _p(centroids), C.c_int32(centroids.shape[0]),
                                 C.c_int32(metric), _p(g))
    return g


def select_clusters(g, w: int):
    g = _c(g, np.float32)
    sel = np.empty(w, np.int32)
    sg = np.empty(w, np.float32)
    lib().oracle_select_clusters(_p(g), C.c_int32(g.shape[0]), C.c_int32(w), _p(sel), _p(sg))
    return sel, sg


def quantize_query(qp):
    qp = _c(qp, np.float32)
    q8 = np.empty(qp.shape[0], np.int8)
    dx = C.c_float(0)
    lib().oracle_quantize_query(_p(qp), C.c_int32(qp.shape[0]), _p(q8), C.byref(dx))
    return q8, np.float32(dx.value)


def stage_a(q8, A_c, dx, dA, dB):
    """A_c is [r][dp] int8.  Returns (R int32 [r], z int8 [r], sigma f32)."""
    q8, A_c = _c(q8, np.int8), _c(A_c, np.int8)
    r, dp = A_c.shape
    R = np.empty(r, np.int32)
    z = np.empty(r, np.int8)
    sg = C.c_float(0)
    lib().oracle_stage_a(_p(q8), C.c_int32(dp), C.c_int32(r), _p(A_c), C.c_float(dx), C.c_float(dA), C.c_float(dB),
                         _p(R), _p(z), C.byref(sg))
    return R, z, np.float32(sg.value)


def stage_a_columns(q8, A_c, dx, dA_cols):
    """Step 4 with one step size per column of A_c.  Returns (R int32 [r], z int8 [r], sigma f32)."""
    q8, A_c, dA_cols = _c(q8, np.int8), _c(A_c, np.int8), _c(dA_cols, np.float32)
    r, dp = A_c.shape
    assert dA_cols.shape == (r,)
    R = np.empty(r, np.int32)
    z = np.empty(r, np.int8)
    sg = C.c_float(0)
    lib().oracle_stage_a_columns(_p(q8), C.c_int32(dp), C.c_int32(r), _p(A_c), C.c_float(dx), _p(dA_cols), _p(R), _p(z),
                                 C.byref(sg))
    return R, z, np.float32(sg.value)


def quantize_query_mixed(qp):
    """Sec. 4.2: the first component stays out of the quantization (code 0 there)."""
    qp = _c(qp, np.float32)
    q8 = np.empty(qp.shape[0], np.int8)
    dx = C.c_float(0)
    lib().oracle_quantize_query_mixed(_p(qp), C.c_int32(qp.shape[0]), _p(q8), C.byref(dx))
    return q8, np.float32(dx.value)


def stage_a_mixed(q8, x0, A_c, dx, dA_cols, A0):
    """Step 4 with the unquantized first component.  Returns (R int32 [r], z int8 [r], sigma f32, rho0 f32)."""
    q8, A_c, dA_cols, A0 = _c(q8, np.int8), _c(A_c, np.int8), _c(dA_cols, np.float32), _c(A0, np.float32)
    r, dp = A_c.shape
    assert dA_cols.shape == (r,) and A0.shape == (r,)
    R = np.empty(r, np.int32)
    z = np.empty(r, np.int8)
    sg, r0 = C.c_float(0), C.c_float(0)
    lib().oracle_stage_a_mixed(_p(q8), C.c_float(x0), C.c_int32(dp), C.c_int32(r), _p(A_c), C.c_float(dx), _p(dA_cols),
                               _p(A0), _p(R), _p(z), C.byref(sg), C.byref(r0))
    return R, z, np.float32(sg.value), np.float32(r0.value)


def score_mixed(Y: int, sigma: float, dB_t: float, rho0: float, B0_t: float, metric: int, sqnorm: float = 0.0) -> np.float32:
    return np.float32(lib().oracle_score_mixed(int(Y), float(sigma), float(dB_t), float(rho0), float(B0_t), int(metric),
                                               float(sqnorm)))


def score_columns(Y: int, sigma: float, dB_t: float, metric: int, sqnorm: float = 0.0) -> np.float32:
    return np.float32(lib().oracle_score_columns(int(Y), float(sigma), float(dB_t), int(metric), float(sqnorm)))


def pair_accumulators(z, B_c):
    """B_c is [m_c][r] int8.  Returns Y int32 [m_c]."""
    z, B_c = _c(z, np.int8), _c(B_c, np.int8)
    Y = np.empty(B_c.shape[0], np.int32)
    lib().oracle_pair_accumulators(_p(z), C.c_int32(B_c.shape[1]), _p(B_c), C.c_int64(B_c.shape[0]), _p(Y))
    return Y


def score(Y: int, sigma: float, metric: int, sqnorm: float = 0.0) -> np.float32:
    return np.float32(lib().oracle_score(int(Y), float(sigma), int(metric), float(sqnorm)))


def row_sqnorm(c) -> np.float32:
    c = _c(c, np.float32)
    return np.float32(lib().oracle_row_sqnorm(_p(c), C.c_int32(c.shape[0])))


def exact_dissim(q, c, metric: int) -> np.float32:
    q, c = _c(q, np.float32), _c(c, np.float32)
    return np.float32(lib().oracle_exact_dissim(_p(q), _p(c), C.c_int32(q.shape[0]), C.c_int32(metric)))


def rrr_predict_f64(x, A, B):
    """Unquantized prediction (x^T A) B in double; A [s][r], B [r][m_c]."""
    x, A, B = _c(x, np.float64), _c(A, np.float64), _c(B, np.float64)
    y = np.empty(B.shape[1], np.float64)
    lib().oracle_rrr_predict_f64(_p(x), C.c_int32(A.shape[0]), C.c_int32(A.shape[1]), _p(A), _p(B),
                                 C.c_int64(B.shape[1]), _p(y))
    return y
