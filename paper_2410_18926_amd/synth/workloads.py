"""The benchmark workloads: shapes, metrics and search parameters of each synthetic configuration.

The shapes follow the data sets of the paper's Table 1 (768-d and 1024-d angular text embeddings, a
1M x 128 Euclidean descriptor set, a 384-d angular set) and the hyper-parameter grid of its Appendix B
(L in {1024, 2048, 4096}, w in {8..256}, candidate-set size in {100..3200}).
"""
from __future__ import annotations

import dataclasses

IP, L2, COS = 0, 1, 2
METRIC_NAMES = {IP: "ip", L2: "l2", COS: "cos"}


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    config_id: int          # enters the seed: seed = 1000 * config_id + stream
    n: int                  # corpus size
    d: int                  # data dimension
    nq: int                 # held-out queries
    G: int                  # mixture components
    alpha: float | None     # power-law exponent of each component's covariance spectrum; None = isotropic
    normalize: bool         # unit-normalise rows
    lognormal_norms: float | None  # sigma of LogNormal(0, sigma) row norms (applied to unit directions)
    metric: int
    L: int                  # clusters
    dp: int                 # reduced dimension d' (== d means P = identity)
    r: int                  # RRR rank
    w: int                  # clusters probed
    m: int                  # candidate-set size (the paper's t)
    k: int = 10
    n_train: int = 200_000  # RRR training sample (drawn from the corpus)
    w_train: int = 16       # routing width used to form each cluster's local training set
    kmeans_iters: int = 10

    def scaled(self, factor: float, name: str | None = None) -> "Workload":
        """A smaller workload with the same per-cluster statistics (n, nq, G, L, n_train scaled together)."""
        f = factor
        return dataclasses.replace(
            self, name=name or f"{self.name}-x{factor:g}", n=max(1, int(self.n * f)),
            nq=max(1, int(self.nq * f)), G=max(1, int(self.G * f)), L=max(1, int(self.L * f)),
            n_train=max(1, int(self.n_train * f)))


WORKLOADS = {
    # C1 Tiny: unit-test size, isotropic mixture, P = I, Euclidean.
    "tiny": Workload("tiny", 1, n=20_000, d=128, nq=1_000, G=64, alpha=None, normalize=False,
                     lognormal_norms=None, metric=L2, L=64, dp=128, r=32, w=8, m=100,
                     n_train=5_000, w_train=8),
    # C2 Embedding-like inner product: the configuration the headline metric is quoted on.
    "embed-ip": Workload("embed-ip", 2, n=1_000_000, d=768, nq=10_000, G=4096, alpha=1.0, normalize=True,
                         lognormal_norms=None, metric=IP, L=1024, dp=256, r=32, w=32, m=200),
    # C3 High-dimensional cosine.
    "highdim-cos": Workload("highdim-cos", 3, n=1_000_000, d=1024, nq=10_000, G=8192, alpha=0.8,
                            normalize=True, lognormal_norms=None, metric=COS, L=2048, dp=256, r=48,
                            w=48, m=300),
    # C4 Low-dimensional squared Euclidean with heavy-tailed norms.
    "lowdim-l2": Workload("lowdim-l2", 4, n=1_000_000, d=128, nq=10_000, G=1024, alpha=1.0, normalize=True,
                          lognormal_norms=0.5, metric=L2, L=1024, dp=128, r=24, w=64, m=200),
    # C5 Scale: 10M x 384.
    "scale-ip": Workload("scale-ip", 5, n=10_000_000, d=384, nq=100_000, G=16384, alpha=1.0, normalize=True,
                         lognormal_norms=None, metric=IP, L=16384, dp=192, r=32, w=64, m=200,
                         n_train=1_000_000),
}


def get_workload(name: str) -> Workload:
    return WORKLOADS[name]
