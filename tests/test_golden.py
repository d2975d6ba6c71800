"""Stored expected values (tests/golden/oracle_search_small.txt, written by tests/golden/make_golden.py from the CPU
oracle alone): the oracle must still reproduce them bit for bit, and the GPU library must return the same neighbours."""
import importlib.util
import pathlib

import numpy as np
import pytest

from oracle import oracle as O

_spec = importlib.util.spec_from_file_location("make_golden", pathlib.Path(__file__).parent / "golden" / "make_golden.py")
G = importlib.util.module_from_spec(_spec)
_spec.loader.exec_module(G)


def _cases():
    for mname, metric in G.METRICS.items():
        for scheme in G.SCHEMES:
            for rerank in (True, False):
                yield mname, metric, scheme, rerank


def test_golden_file_is_complete():
    stored = G.read_golden()
    assert sorted(stored) == sorted(G.case_name(m, s, r) for m, _, s, r in _cases())
    for ids, dists in stored.values():
        assert ids.shape == (G.NQ, G.K) and dists.shape == (G.NQ, G.K)
        assert (ids >= 0).all() and np.isfinite(dists).all()
        assert (np.diff(dists, axis=1) >= 0).all()              # nearest first


def test_oracle_reproduces_the_stored_values():
    """A change of the oracle's arithmetic shows here; it needs the passage that justifies it and a regenerated file."""
    stored = G.read_golden()
    for mname, metric, scheme, rerank in _cases():
        ix, q = G.golden_index(metric, scheme)
        oix = O.OracleIndex(ix)
        ids, dists = O.search(oix, q, G.K, G.W, G.M) if rerank else O.search_no_rerank(oix, q, G.K, G.W)
        s_ids, s_d = stored[G.case_name(mname, scheme, rerank)]
        np.testing.assert_array_equal(ids, s_ids, err_msg=G.case_name(mname, scheme, rerank))
        np.testing.assert_array_equal(dists.view(np.uint32), s_d.view(np.uint32), err_msg=G.case_name(mname, scheme, rerank))


def test_stored_values_distinguish_the_schemes_and_modes():
    """The fixture is only worth something if its cases differ: the three quantization schemes give different
    neighbour lists on their inputs, and leaving out the re-ranking changes the answer."""
    stored = G.read_golden()
    for mname in G.METRICS:
        with_rr = [stored[G.case_name(mname, s, True)][0] for s in G.SCHEMES]
        assert not np.array_equal(with_rr[0], with_rr[1]) and not np.array_equal(with_rr[1], with_rr[2])
        for s in G.SCHEMES:
            assert not np.array_equal(stored[G.case_name(mname, s, True)][0], stored[G.case_name(mname, s, False)][0])


@pytest.mark.gpu
def test_library_matches_the_stored_values():
    from paper_2410_18926_amd import binding as B
    from tests.parity_util import assert_topk_equal
    stored = G.read_golden()
    for mname, metric, scheme, rerank in _cases():
        ix, q = G.golden_index(metric, scheme)
        gix = B.Index(**ix)
        if not rerank:
            gix.set_rerank(B.RERANK_NONE)
        ids, dists = gix.search(q, G.K, G.W, G.M if rerank else G.K)
        s_ids, s_d = stored[G.case_name(mname, scheme, rerank)]
        if rerank:
            assert_topk_equal(ids, dists, s_ids, s_d, G.case_name(mname, scheme, rerank))
        else:       # estimated scores: every operation is specified, the results are bit-identical
            np.testing.assert_array_equal(ids, s_ids, err_msg=G.case_name(mname, scheme, rerank))
            np.testing.assert_array_equal(dists, s_d, err_msg=G.case_name(mname, scheme, rerank))
        gix.close()
