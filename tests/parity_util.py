"""Comparison helpers shared by the GPU parity tests."""
import numpy as np

DIST_RTOL = 1e-4      # float re-rank distances: GPU accumulates in fp32, the oracle in fp64
TIE_RTOL = 1e-5       # returned ids may differ only where the distances tie within this relative tolerance


def assert_topk_equal(ids_gpu, dists_gpu, ids_ref, dists_ref, what="", floor=1e-3):
    """ids identical except at ties within TIE_RTOL; distances within DIST_RTOL (relative, with an absolute floor
    for distances near zero: an inner product that cancels to almost nothing carries the float rounding of its
    terms, so callers whose results include such values pass a floor on the scale of |q| |x|)."""
    ids_gpu, ids_ref = np.asarray(ids_gpu), np.asarray(ids_ref)
    dists_gpu, dists_ref = np.asarray(dists_gpu, np.float64), np.asarray(dists_ref, np.float64)
    assert ids_gpu.shape == ids_ref.shape and dists_gpu.shape == dists_ref.shape, what
    pad = ids_ref < 0
    assert np.array_equal(pad, ids_gpu < 0), f"{what}: padding differs"
    assert np.all(np.isinf(dists_gpu[pad])), what
    ok = ~pad
    scale = np.maximum(np.abs(dists_ref[ok]), floor)
    err = np.abs(dists_gpu[ok] - dists_ref[ok]) / scale
    assert err.size == 0 or err.max() <= DIST_RTOL, f"{what}: distance error {err.max():.3g}"
    mism = ok & (ids_gpu != ids_ref)
    if mism.any():
        # every mismatching position must be a tie: the same distance (within tolerance) on both sides,
        # and per query the multisets of ids may differ only among tied entries
        for qi in np.unique(np.nonzero(mism)[0]):
            cols = np.nonzero(mism[qi])[0]
            for c in cols:
                near = np.abs(dists_ref[qi] - dists_ref[qi, c]) <= TIE_RTOL * max(abs(dists_ref[qi, c]), floor)
                partner_ok = ids_gpu[qi, c] in ids_ref[qi][near] or c == ids_ref.shape[1] - 1 or near[-1]
                assert partner_ok, f"{what}: query {qi} position {c}: id {ids_gpu[qi, c]} vs {ids_ref[qi, c]} is not a tie"
    return int(mism.sum())


def y_offsets(sel, cluster_offsets):
    """Offsets of every (query, rank) slot into the flat integer-score dump."""
    sizes = (cluster_offsets[1:] - cluster_offsets[:-1])[sel.reshape(-1)]
    off = np.zeros(sizes.size + 1, np.int64)
    np.cumsum(sizes, out=off[1:])
    return off
