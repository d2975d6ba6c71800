"""Seeded Gaussian-mixture corpora and held-out query batches.

Stand-ins for the public data sets the paper evaluates on (its Table 1: unit-norm text/image embeddings of
384-1536 dimensions, and 128-d Euclidean descriptors), with their shapes and the low intrinsic
dimensionality typical of embeddings.  Nothing here belongs to the search method.

Recipe (seed = 1000 * config_id + stream):
  * G mixture components with uniform weights; component means mu_g ~ N(0, 4 I).
  * isotropic workloads: x = mu_g + xi, xi ~ N(0, I).
  * anisotropic workloads: x = mu_g + U (sqrt(lambda)[pi_g] * xi); lambda_i proportional to i^-alpha and
    normalised to mean 1; U is one seeded orthogonal matrix shared by all components (QR of a Gaussian
    matrix); pi_g is a seeded permutation per component that assigns the spectrum to the axes, so every
    component has its own covariance without G dense d x d matrices being stored.
  * optional unit normalisation of the rows, optional LogNormal(0, sigma) row norms applied afterwards.
  * queries are further draws from the same mixture with an independent stream.
"""
from __future__ import annotations

import math

import torch

from .workloads import Workload

_STREAM_MEANS, _STREAM_BASIS, _STREAM_PERM, _STREAM_CORPUS, _STREAM_QUERIES = 1, 2, 3, 4, 5


def _gen(device: torch.device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


class _Mixture:
    def __init__(self, wl: Workload, device: torch.device):
        self.wl, self.device = wl, device
        base = 1000 * wl.config_id
        d, G = wl.d, wl.G
        self.means = 2.0 * torch.randn(G, d, generator=_gen(device, base + _STREAM_MEANS), device=device)
        if wl.alpha is not None:
            lam = torch.arange(1, d + 1, dtype=torch.float64) ** (-wl.alpha)
            lam = lam * (d / lam.sum())
            self.sqrt_lam = lam.sqrt().to(torch.float32).to(device)
            a = torch.randn(d, d, generator=_gen(device, base + _STREAM_BASIS), device=device)
            q, r = torch.linalg.qr(a.cpu().double())
            q = q * torch.sign(torch.diagonal(r)).unsqueeze(0)
            self.U = q.to(torch.float32).to(device)
            # per-component permutation of the spectrum over the axes: argsort of seeded uniforms
            u = torch.rand(G, d, generator=_gen(device, base + _STREAM_PERM), device=device)
            self.perm = torch.argsort(u, dim=1)
        else:
            self.sqrt_lam = self.U = self.perm = None

    def draw(self, count: int, stream: int, chunk: int = 131072) -> torch.Tensor:
        wl, dev = self.wl, self.device
        g = _gen(dev, 1000 * wl.config_id + stream)
        out = torch.empty(count, wl.d, dtype=torch.float32, device=dev)
        for s in range(0, count, chunk):
            e = min(count, s + chunk)
            comp = torch.randint(0, wl.G, (e - s,), generator=g, device=dev)
            xi = torch.randn(e - s, wl.d, generator=g, device=dev)
            if self.U is not None:
                xi = (xi * self.sqrt_lam[self.perm[comp]]) @ self.U.T
            x = self.means[comp] + xi
            if wl.normalize:
                x = x / x.norm(dim=1, keepdim=True)
            if wl.lognormal_norms is not None:
                z = torch.randn(e - s, 1, generator=g, device=dev)
                x = x * torch.exp(wl.lognormal_norms * z)
            out[s:e] = x
        return out


def make_dataset(wl: Workload, device: str | torch.device = "cpu", nq: int | None = None, extra_batches: int = 0):
    """Return (corpus [n, d] fp32, queries [nq, d] fp32) on `device` for workload `wl`.

    With extra_batches > 0 a third value is returned: a list of further, distinct query batches of the same
    size (independent streams), for timing loops that must not repeat a batch.

    The values depend on the device type (torch's CPU and GPU generators are different streams); a given
    device type always reproduces the same arrays.
    """
    device = torch.device(device)
    mix = _Mixture(wl, device)
    corpus = mix.draw(wl.n, _STREAM_CORPUS)
    count = wl.nq if nq is None else nq
    queries = mix.draw(count, _STREAM_QUERIES)
    if extra_batches <= 0:
        return corpus, queries
    extra = [mix.draw(count, _STREAM_QUERIES + 1 + b) for b in range(extra_batches)]
    return corpus, queries, extra


def draw_queries(wl: Workload, device: str | torch.device, count: int, batch_index: int) -> torch.Tensor:
    """`count` held-out queries of workload `wl` from the stream of query batch `batch_index` (0 = the batch
    make_dataset returns, 1.. = its extra batches; any larger index is a further independent stream)."""
    device = torch.device(device)
    return _Mixture(wl, device).draw(count, _STREAM_QUERIES + batch_index)


def brute_force_topk(corpus: torch.Tensor, queries: torch.Tensor, metric: int, k: int, chunk: int | None = None):
    """Ground-truth neighbours by exhaustive fp32 scoring (used for recall only, never timed).

    Returns (ids [nq, k] int64, dists [nq, k] fp32) with the paper's dissimilarities: squared L2,
    negative inner product, or 1 - cosine.
    """
    from .workloads import IP, L2, COS
    nq = queries.shape[0]
    if chunk is None:       # keep the [chunk, n] score block near 2^31 elements (8 GiB) whatever the corpus size
        chunk = int(max(16, min(2048, (1 << 31) // max(1, corpus.shape[0]))))
    ids = torch.empty(nq, k, dtype=torch.int64, device=queries.device)
    dists = torch.empty(nq, k, dtype=torch.float32, device=queries.device)
    cn = (corpus * corpus).sum(1) if metric == L2 else None
    for s in range(0, nq, chunk):
        q = queries[s:s + chunk]
        ip = q @ corpus.T
        if metric == IP:
            dis = -ip
        elif metric == L2:
            dis = (q * q).sum(1, keepdim=True) - 2 * ip + cn.unsqueeze(0)
        else:
            dis = 1 - ip / q.norm(dim=1, keepdim=True) / corpus.norm(dim=1).unsqueeze(0)
        v, i = torch.topk(dis, k, dim=1, largest=False)
        ids[s:s + chunk], dists[s:s + chunk] = i, v
    return ids, dists
