"""Index construction for the synthetic workloads: the arrays `lorann_load_index` (and the CPU oracle) take.

Index construction is not on the query-phase hot path; it is input preparation written with plain torch
ops so that it runs on the CPU (unit-test sizes) and on the GPU (million-point corpora) alike.  It follows
the paper's index phase:

  * Sec. 4.1: projection matrix = the first d' eigenvectors of the uncentered second-moment matrix of the
    training set; k-means on the projected corpus; centroids live in the d'-dimensional space.
  * Sec. 2.2: standard k-means for Euclidean distance, spherical k-means for inner product / cosine.
  * Sec. 3.2 + 4.1: per cluster, local training set = training points that have the cluster among their
    w_train nearest centroids; Y = X C^T (true d-dimensional inner products); V_r = first r right singular
    vectors of Y; A = (X W_s)^+ Y V_r, B = V_r^T (without dimensionality reduction this is A = C^T V_r when
    X has full column rank).
  * Sec. 3.3 / 4.2: random rotations folded into the projection and into V_r; absmax 8-bit quantization.
    The scale granularity is one scalar per cluster for A and one for B (the format this library's
    boundary fixes), stored as the step size Delta = max|.| / 127.
"""
from __future__ import annotations

import dataclasses

import torch

from .workloads import IP, L2, COS, Workload


@dataclasses.dataclass
class IndexArrays:
    """Arrays in exactly the layout of `lorann_load_index` (all torch tensors, same device)."""
    metric: int
    n: int
    d: int
    dp: int
    r: int
    L: int
    centroids: torch.Tensor        # [L, dp] f32
    P: torch.Tensor | None         # [d, dp] f32 row-major, None = identity
    A: torch.Tensor                # [L, r, dp] int8   (A_c transposed: d' contiguous)
    B: torch.Tensor                # [n, r] int8       (one r-byte code per point, rows in cluster order)
    scale_A: torch.Tensor          # [L] f32  Delta_A: real A ~= Delta_A[c] * A_i8
    scale_B: torch.Tensor          # [L] f32
    cluster_offsets: torch.Tensor  # [L + 1] int64
    corpus: torch.Tensor           # [n, d] f32, rows in cluster order
    ids: torch.Tensor              # [n] int64: original index of each row
    scale_A_columns: torch.Tensor | None = None   # [L, r] f32: one step size per column of A_c (Sec. 3.3 as printed);
    scale_B_points: torch.Tensor | None = None    # [n] f32: one per column of B_c, i.e. per corpus row; both or neither
    first_row_A: torch.Tensor | None = None       # [L, r] f32: A_c[0][j] unquantized (Sec. 4.2 mixed precision); with
    first_row_B: torch.Tensor | None = None       # [n] f32: B_c[0][t] unquantized; both or neither, need the column scales
    A_f32: torch.Tensor | None = None   # [L, r, dp] unquantized factors (kept on request, for tests)
    B_f32: torch.Tensor | None = None   # [n, r]

    def to(self, device) -> "IndexArrays":
        kw = {}
        for f in dataclasses.fields(self):
            v = getattr(self, f.name)
            kw[f.name] = v.to(device) if isinstance(v, torch.Tensor) else v
        return IndexArrays(**kw)

    def numpy(self) -> dict:
        out = {}
        for f in dataclasses.fields(self):
            v = getattr(self, f.name)
            out[f.name] = v.detach().cpu().contiguous().numpy() if isinstance(v, torch.Tensor) else v
        return out


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _random_rotation(dim: int, seed: int, device) -> torch.Tensor:
    a = torch.randn(dim, dim, generator=_gen("cpu", seed), dtype=torch.float64)
    q, r = torch.linalg.qr(a)
    return (q * torch.sign(torch.diagonal(r)).unsqueeze(0)).to(device)


def _route(xp: torch.Tensor, centroids: torch.Tensor, metric: int, w: int, chunk: int = 65536) -> torch.Tensor:
    """w nearest centroids of each projected point (ids only)."""
    out = torch.empty(xp.shape[0], w, dtype=torch.int64, device=xp.device)
    cn = (centroids * centroids).sum(1) if metric == L2 else None
    for s in range(0, xp.shape[0], chunk):
        ip = xp[s:s + chunk] @ centroids.T
        g = (cn.unsqueeze(0) - 2 * ip) if metric == L2 else -ip
        out[s:s + chunk] = torch.topk(g, w, dim=1, largest=False).indices
    return out


def _kmeans(xp: torch.Tensor, L: int, metric: int, iters: int, seed: int):
    n = xp.shape[0]
    init = torch.randperm(n, generator=_gen("cpu", seed))[:L].to(xp.device)
    cent = xp[init].clone()
    spherical = metric != L2
    if spherical:
        cent = cent / cent.norm(dim=1, keepdim=True).clamp_min(1e-30)
    for _ in range(iters):
        assign = _route(xp, cent, metric, 1).squeeze(1)
        sums = torch.zeros_like(cent).index_add_(0, assign, xp)
        cnt = torch.zeros(L, device=xp.device, dtype=xp.dtype).index_add_(0, assign, torch.ones_like(assign, dtype=xp.dtype))
        new = sums / cnt.clamp_min(1).unsqueeze(1)
        if spherical:
            new = new / new.norm(dim=1, keepdim=True).clamp_min(1e-30)
        cent = torch.where((cnt > 0).unsqueeze(1), new, cent)   # an empty cluster keeps its centroid
    assign = _route(xp, cent, metric, 1).squeeze(1)
    return cent, assign


def _top_right_singular(Y: torch.Tensor, r: int, exact: bool, seed: int) -> torch.Tensor:
    """First min(r, rank-bound) right singular vectors of Y [n_l, m_l] as columns [m_l, r'] (r' <= r)."""
    n_l, m_l = Y.shape
    rr = min(r, n_l, m_l)
    if rr == 0:
        return Y.new_zeros(m_l, 0)
    q = min(m_l, n_l, r + 16)
    if exact or q >= min(n_l, m_l):
        _, _, vh = torch.linalg.svd(Y, full_matrices=False)
        return vh[:rr].T.contiguous()
    # randomized range finder with power iterations (Halko et al.), as the paper does in practice
    omega = torch.randn(m_l, q, generator=_gen("cpu", seed), dtype=torch.float64).to(Y.device, Y.dtype)
    Q, _ = torch.linalg.qr(Y.T @ (Y @ omega))
    for _ in range(3):
        Q, _ = torch.linalg.qr(Y.T @ (Y @ Q))
    T = Y @ Q                                     # [n_l, q]
    _, _, wh = torch.linalg.svd(T, full_matrices=False)
    return (Q @ wh[:rr].T).contiguous()


def _absmax_int8(x: torch.Tensor):
    """Absmax quantization with one scalar for the whole array: (codes int8, Delta = max|x| / 127)."""
    a = x.abs().max() if x.numel() else x.new_zeros(())
    if float(a) == 0.0:
        return torch.zeros_like(x, dtype=torch.int8), 0.0
    delta = (a / 127.0).to(torch.float32)
    codes = torch.round(x.to(torch.float32) / delta).clamp_(-127, 127).to(torch.int8)
    return codes, float(delta)


def _absmax_int8_rows(x: torch.Tensor):
    """Absmax quantization with one scalar per row of x [rows, len]: (codes int8, Delta [rows] = max|row| / 127)."""
    a = x.abs().amax(dim=1).to(torch.float32)
    delta = a / 127.0
    safe = torch.where(delta > 0, delta, torch.ones_like(delta))
    codes = torch.round(x.to(torch.float32) / safe[:, None]).clamp_(-127, 127).to(torch.int8)
    codes[delta == 0] = 0
    return codes, delta


def build_index(corpus: torch.Tensor, wl: Workload, *, exact_svd: bool = False, rotate: bool = True,
                keep_float: bool = False, fit_dtype: torch.dtype = torch.float64,
                train: torch.Tensor | None = None, progress=None, column_scales: bool = False,
                mixed_precision: bool = False) -> IndexArrays:
    """Build the index arrays for `corpus` [n, d] under workload `wl` on corpus.device.

    `train` overrides the RRR training set (default: a seeded sample of min(n, wl.n_train) corpus rows).
    `column_scales`: quantize every column of A_c and of B_c with its own step size (Sec. 3.3 as printed) instead
    of one step size per cluster and matrix; the codes differ, and scale_A / scale_B then only hold the largest of
    the column step sizes (the search ignores them once the column scales are set).
    `mixed_precision` (Sec. 4.2; implies column_scales): the first row of every A_c and B_c is kept in float
    (first_row_A, first_row_B), its codes are zero and the step sizes come from the other rows alone; the random
    rotations then leave the first component (the principal axis, the leading singular direction) in place.
    """
    column_scales = column_scales or mixed_precision
    dev = corpus.device
    n, d = corpus.shape
    dp, r, L, metric = wl.dp, wl.r, wl.L, wl.metric
    base = 1000 * wl.config_id
    say = progress or (lambda *_: None)

    if train is None:
        nt = min(n, wl.n_train)
        tsel = torch.randperm(n, generator=_gen("cpu", base + 11))[:nt].to(dev)
        train = corpus[tsel]

    # ---- projection (Sec. 4.1) with a random rotation folded in (Sec. 4.2) ----
    if dp == d:
        P = None
    else:
        gram = torch.zeros(d, d, dtype=torch.float64, device=dev)
        for s in range(0, train.shape[0], 65536):
            t = train[s:s + 65536].double()
            gram += t.T @ t
        evals, evecs = torch.linalg.eigh(gram.cpu())
        W = evecs[:, torch.argsort(evals, descending=True)[:dp]]          # [d, dp] fp64
        if rotate and mixed_precision:
            W = torch.cat([W[:, :1], W[:, 1:] @ _random_rotation(dp - 1, base + 12, "cpu")], 1)
        elif rotate:
            W = W @ _random_rotation(dp, base + 12, "cpu")
        P = W.to(torch.float32).to(dev).contiguous()
    say("projection done")

    def project(x):
        return x if P is None else x @ P

    # ---- clustering in the projected space (Sec. 4.1, 2.2) ----
    xp = torch.empty(n, dp, dtype=torch.float32, device=dev)
    for s in range(0, n, 131072):
        xp[s:s + 131072] = project(corpus[s:s + 131072])
    centroids, assign = _kmeans(xp, L, metric, wl.kmeans_iters, base + 13)
    del xp
    order = torch.argsort(assign, stable=True)
    counts = torch.bincount(assign, minlength=L)
    offsets = torch.zeros(L + 1, dtype=torch.int64, device=dev)
    offsets[1:] = torch.cumsum(counts, 0)
    corpus_sorted = corpus[order].contiguous()
    say("clustering done")

    # ---- local training sets (Sec. 3.2) ----
    w_train = min(wl.w_train, L)
    tp = project(train)
    tr_route = _route(tp, centroids, metric, w_train)                      # [nt, w_train]
    flat_c = tr_route.reshape(-1)
    flat_i = torch.arange(train.shape[0], device=dev).repeat_interleave(w_train)
    o = torch.argsort(flat_c, stable=True)
    tr_members = flat_i[o]
    tr_off = torch.zeros(L + 1, dtype=torch.int64, device=dev)
    tr_off[1:] = torch.cumsum(torch.bincount(flat_c, minlength=L), 0)
    tr_off_h, off_h = tr_off.tolist(), offsets.tolist()

    A_q = torch.zeros(L, r, dp, dtype=torch.int8, device=dev)
    B_q = torch.zeros(n, r, dtype=torch.int8, device=dev)
    sA = torch.zeros(L, dtype=torch.float32)
    sB = torch.zeros(L, dtype=torch.float32)
    sA_cols = torch.zeros(L, r, dtype=torch.float32, device=dev) if column_scales else None
    sB_pts = torch.zeros(n, dtype=torch.float32, device=dev) if column_scales else None
    A_first = torch.zeros(L, r, dtype=torch.float32, device=dev) if mixed_precision else None
    B_first = torch.zeros(n, dtype=torch.float32, device=dev) if mixed_precision else None
    A_f = torch.zeros(L, r, dp, dtype=torch.float32, device=dev) if keep_float else None
    B_f = torch.zeros(n, r, dtype=torch.float32, device=dev) if keep_float else None
    Pd = None if P is None else P.to(fit_dtype)

    for l in range(L):
        c0, c1 = off_h[l], off_h[l + 1]
        m_l = c1 - c0
        if m_l == 0:
            continue
        C = corpus_sorted[c0:c1].to(fit_dtype)
        X = train[tr_members[tr_off_h[l]:tr_off_h[l + 1]]].to(fit_dtype)
        if X.shape[0] < dp:                      # too few routed training points: add the cluster's own points
            X = torch.cat([X, C], 0)
        Xt = X if Pd is None else X @ Pd
        Y = X @ C.T                                                        # [n_l, m_l]
        V = _top_right_singular(Y, r, exact_svd, base + 100 + l)           # [m_l, r']
        rr = V.shape[1]
        if rotate and mixed_precision and rr > 2:
            V = torch.cat([V[:, :1], V[:, 1:] @ _random_rotation(rr - 1, base + 14, dev).to(fit_dtype)], 1)
        elif rotate and rr > 1 and not mixed_precision:
            V = V @ _random_rotation(rr, base + 14, dev).to(fit_dtype)
        YV = Y @ V                                                         # [n_l, r']
        # A = Xt^+ (Y V): least squares through the normal equations with a tiny ridge for rank safety
        G = Xt.T @ Xt
        ridge = 1e-9 * torch.trace(G) / dp
        G = G + ridge * torch.eye(dp, dtype=fit_dtype, device=dev)
        A = torch.linalg.solve(G, Xt.T @ YV)                               # [dp, r']
        Af = torch.zeros(r, dp, dtype=torch.float32, device=dev)
        Bf = torch.zeros(m_l, r, dtype=torch.float32, device=dev)
        Af[:rr] = A.T.to(torch.float32)
        Bf[:, :rr] = V.to(torch.float32)
        if mixed_precision:
            A_first[l], B_first[c0:c1] = Af[:, 0], Bf[:, 0]
            A_q[l, :, 1:], sA_cols[l] = _absmax_int8_rows(Af[:, 1:])
            B_q[c0:c1, 1:], sB_pts[c0:c1] = _absmax_int8_rows(Bf[:, 1:])
            sA[l], sB[l] = float(sA_cols[l].max()), float(sB_pts[c0:c1].max())
        elif column_scales:
            A_q[l], sA_cols[l] = _absmax_int8_rows(Af)          # rows of A_c^T are the columns of A_c
            B_q[c0:c1], sB_pts[c0:c1] = _absmax_int8_rows(Bf)    # rows of B_c^T are the columns of B_c
            sA[l], sB[l] = float(sA_cols[l].max()), float(sB_pts[c0:c1].max())
        else:
            A_q[l], sA[l] = _absmax_int8(Af)
            B_q[c0:c1], sB[l] = _absmax_int8(Bf)
        if keep_float:
            A_f[l], B_f[c0:c1] = Af, Bf
        if (l + 1) % 128 == 0:
            say(f"fit {l + 1}/{L}")

    return IndexArrays(metric=metric, n=n, d=d, dp=dp, r=r, L=L, centroids=centroids.contiguous(), P=P,
                       A=A_q, B=B_q, scale_A=sA.to(dev), scale_B=sB.to(dev), cluster_offsets=offsets,
                       corpus=corpus_sorted, ids=order.to(torch.int64).contiguous(), scale_A_columns=sA_cols,
                       scale_B_points=sB_pts, first_row_A=A_first, first_row_B=B_first, A_f32=A_f, B_f32=B_f)


def random_index(corpus: torch.Tensor, wl: Workload) -> IndexArrays:
    """Index arrays of the right shapes with RANDOM content (unit random centroids, uniform random int8 factors
    and codes, clusters of 0.65..1.35 times the mean size cut from the corpus in its given order).

    Search results on it mean nothing.  It exists to time and profile kernels whose cost does not depend on the
    values (the streaming of the codes, the row gather) at shapes whose real index takes minutes to fit.
    """
    dev = corpus.device
    n, d = corpus.shape
    dp, r, L = wl.dp, wl.r, wl.L
    g = _gen(dev, 1000 * wl.config_id + 77)
    cent = torch.randn(L, dp, generator=g, device=dev)
    cent = cent / cent.norm(dim=1, keepdim=True)
    sizes = 0.65 + 0.7 * torch.rand(L, generator=g, device=dev, dtype=torch.float64)
    sizes = torch.floor(sizes * (n / sizes.sum())).long()
    sizes[0] += n - sizes.sum()
    offsets = torch.zeros(L + 1, dtype=torch.int64, device=dev)
    offsets[1:] = torch.cumsum(sizes, 0)
    P = None
    if dp != d:
        P = _random_rotation(d, 1000 * wl.config_id + 78, "cpu")[:, :dp].to(torch.float32).to(dev).contiguous()
    A = torch.randint(-127, 128, (L, r, dp), generator=g, device=dev, dtype=torch.int8)
    B = torch.randint(-127, 128, (n, r), generator=g, device=dev, dtype=torch.int8)
    s = torch.full((L,), 1e-3, device=dev)
    return IndexArrays(metric=wl.metric, n=n, d=d, dp=dp, r=r, L=L, centroids=cent, P=P, A=A, B=B, scale_A=s,
                       scale_B=s.clone(), cluster_offsets=offsets, corpus=corpus,
                       ids=torch.arange(n, dtype=torch.int64, device=dev))
