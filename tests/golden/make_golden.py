"""Writes tests/golden/oracle_search_small.txt: results of the CPU oracle on a small, fully deterministic index.

    python tests/golden/make_golden.py          (from the repository root; overwrites the file)

The values are produced by `oracle/` alone.  The inputs are generated here from integer draws of a seeded numpy
generator, scaled by powers of two, so they are identical on every machine and need no fitted index.  The file pins the
oracle against silent changes of its arithmetic (a change must come with the passage of the paper that justifies it
and a regenerated file) and serves as stored expected values for the GPU library.

Cases: the three dissimilarities (Sec. 2.1) x the three quantization schemes (one step size per cluster; Sec. 3.3
column-wise step sizes; Sec. 4.2 mixed-precision decomposition) x with / without the final re-ranking step (Sec. 2.2,
App. D.3).
"""
from __future__ import annotations

import pathlib
import sys

import numpy as np

ROOT = pathlib.Path(__file__).resolve().parents[2]
GOLDEN = pathlib.Path(__file__).resolve().parent / "oracle_search_small.txt"
METRICS = {"ip": 0, "l2": 1, "cos": 2}
SCHEMES = ("cluster", "columns", "mixed")
K, W, M, NQ = 5, 4, 25, 12


def golden_index(metric: int, scheme: str) -> tuple[dict, np.ndarray]:
    """(index dict in the layout of the load call, queries [NQ, d]).  Integer draws and dyadic scales only."""
    g = np.random.default_rng(2410_18926 + 10 * metric + SCHEMES.index(scheme))
    n, d, dp, r, L = 640, 24, 16, 8, 12
    cuts = np.sort(g.choice(np.arange(1, n), size=L - 1, replace=False))
    off = np.concatenate([[0], cuts, [n]]).astype(np.int64)
    corpus = (g.integers(-24, 25, size=(n, d)) / 8.0).astype(np.float32)
    P = (g.integers(-4, 5, size=(d, dp)) / 8.0).astype(np.float32)
    ix = dict(metric=metric, n=n, d=d, dp=dp, r=r, L=L,
              centroids=(g.integers(-40, 41, size=(L, dp)) / 4.0).astype(np.float32), P=P,
              A=g.integers(-127, 128, size=(L, r, dp)).astype(np.int8),
              B=g.integers(-127, 128, size=(n, r)).astype(np.int8),
              scale_A=(2.0 ** g.integers(-9, -5, size=L)).astype(np.float32),
              scale_B=(2.0 ** g.integers(-9, -5, size=L)).astype(np.float32),
              cluster_offsets=off, corpus=corpus, ids=g.permutation(n).astype(np.int64))
    if scheme in ("columns", "mixed"):
        ix["scale_A_columns"] = (2.0 ** g.integers(-10, -4, size=(L, r))).astype(np.float32)
        ix["scale_B_points"] = (2.0 ** g.integers(-10, -4, size=n)).astype(np.float32)
    if scheme == "mixed":
        ix["first_row_A"] = (g.integers(-16, 17, size=(L, r)) / 8.0).astype(np.float32)
        ix["first_row_B"] = (g.integers(-16, 17, size=n) / 8.0).astype(np.float32)
    queries = (g.integers(-24, 25, size=(NQ, d)) / 8.0).astype(np.float32)
    return ix, queries


def case_name(metric_name: str, scheme: str, rerank: bool) -> str:
    return f"metric={metric_name} scheme={scheme} rerank={int(rerank)}"


def format_case(ids: np.ndarray, dists: np.ndarray) -> list[str]:
    """One line per query: the k ids, then the k distances as the hexadecimal bit patterns of their floats."""
    bits = np.ascontiguousarray(dists, np.float32).view(np.uint32)
    return [" ".join(str(int(v)) for v in ids[q]) + " | " + " ".join(f"{int(b):08x}" for b in bits[q]) for q in range(ids.shape[0])]


def read_golden() -> dict:
    """{case name: (ids int64 [NQ, K], dists float32 [NQ, K])}"""
    out, name, rows = {}, None, []

    def flush():
        if name is not None:
            ids = np.array([[int(v) for v in r.split("|")[0].split()] for r in rows], np.int64)
            bits = np.array([[int(v, 16) for v in r.split("|")[1].split()] for r in rows], np.uint32)
            out[name] = (ids, bits.view(np.float32))

    for line in GOLDEN.read_text().splitlines():
        if line.startswith("#") or not line.strip():
            continue
        if line.startswith("case "):
            flush()
            name, rows = line[5:].strip(), []
        else:
            rows.append(line)
    flush()
    return out


def main() -> None:
    sys.path.insert(0, str(ROOT))
    from oracle import oracle as O
    lines = ["# Written by tests/golden/make_golden.py from the CPU oracle alone (see that file).",
             f"# k={K} w={W} m={M} queries={NQ}; per query: ids | float32 bit patterns of the distances",
             "# Passages: Sec. 2.1 (dissimilarities), Sec. 2.2 (candidates, re-ranking), Sec. 3.2-3.3 (8-bit scores),",
             "# Sec. 4.1 (projection), Sec. 4.2 (mixed-precision decomposition), App. D.3 (no re-ranking)."]
    for mname, metric in METRICS.items():
        for scheme in SCHEMES:
            ix, q = golden_index(metric, scheme)
            oix = O.OracleIndex(ix)
            for rerank in (True, False):
                ids, dists = O.search(oix, q, K, W, M) if rerank else O.search_no_rerank(oix, q, K, W)
                lines.append("case " + case_name(mname, scheme, rerank))
                lines += format_case(ids, dists)
    GOLDEN.write_text("\n".join(lines) + "\n")
    print(f"wrote {GOLDEN} ({len(lines)} lines)")


if __name__ == "__main__":
    main()
