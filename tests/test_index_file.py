"""The serialized index file: the Python writer, the oracle's C reader and the library's reader agree."""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2410_18926_amd.synth.index_file import save_index, read_index


def _index(rng, metric, with_P, with_ids):
    n, d, L, r = 400, 32, 7, 8
    dp = 16 if with_P else d
    cuts = np.sort(rng.choice(np.arange(1, n), size=L - 1, replace=False))
    corpus = rng.normal(size=(n, d)).astype(np.float32)
    return dict(metric=metric, n=n, d=d, dp=dp, r=r, L=L, centroids=rng.normal(size=(L, dp)).astype(np.float32),
                P=np.linalg.qr(rng.normal(size=(d, d)))[0][:, :dp].astype(np.float32) if with_P else None,
                A=rng.integers(-127, 128, size=(L, r, dp)).astype(np.int8), B=rng.integers(-127, 128, size=(n, r)).astype(np.int8),
                scale_A=rng.uniform(0.01, 0.1, L).astype(np.float32), scale_B=rng.uniform(0.01, 0.1, L).astype(np.float32),
                cluster_offsets=np.concatenate([[0], cuts, [n]]).astype(np.int64), corpus=corpus,
                ids=rng.permutation(n).astype(np.int64) + 1000 if with_ids else None)


@pytest.mark.parametrize("metric,with_P,with_ids", [(0, True, True), (1, False, False), (2, True, False), (1, False, True)])
def test_round_trip_and_oracle_reader(tmp_path, metric, with_P, with_ids):
    rng = np.random.default_rng(10 * metric + with_P + 2 * with_ids)
    ix = _index(rng, metric, with_P, with_ids)
    path = tmp_path / "index.lrn"
    save_index(path, ix)
    back = read_index(path)
    for k, v in ix.items():
        if isinstance(v, np.ndarray):
            np.testing.assert_array_equal(np.asarray(back[k]), v, err_msg=k)
        else:
            assert back[k] == v, k
    # every array starts at a multiple of 64 bytes
    assert all(np.asarray(back[k]).ctypes.data % 64 == np.asarray(back["cluster_offsets"]).ctypes.data % 64
               for k in ("centroids", "A", "B", "scale_A", "scale_B", "corpus"))
    # the oracle's own reader gives an index that searches exactly like the one built from the arrays
    q = rng.normal(size=(25, ix["d"])).astype(np.float32)
    a_ids, a_d, a_st = O.search(O.OracleIndex(ix), q, 5, 3, 40, stages=True)
    f_ids, f_d, f_st = O.search(O.OracleIndex.from_file(path), q, 5, 3, 40, stages=True)
    np.testing.assert_array_equal(f_ids, a_ids)
    np.testing.assert_array_equal(f_d, a_d)
    for k in a_st:
        np.testing.assert_array_equal(f_st[k], a_st[k], err_msg=k)


def test_bad_files_are_refused(tmp_path):
    rng = np.random.default_rng(3)
    ix = _index(rng, 0, True, True)
    good = tmp_path / "good.lrn"
    save_index(good, ix)
    data = good.read_bytes()
    short = tmp_path / "short.lrn"
    short.write_bytes(data[:len(data) - 100])
    foreign = tmp_path / "foreign.lrn"
    foreign.write_bytes(b"NOTANIDX" + data[8:])
    for p in (short, foreign, tmp_path / "missing.lrn"):
        with pytest.raises(ValueError):
            O.OracleIndex.from_file(p)
    with pytest.raises(ValueError):
        read_index(foreign)
    # the library refuses them before touching the GPU
    from paper_2410_18926_amd import binding
    if not binding.LIB_PATH.exists():
        pytest.skip("HIP library not built")
    for p in (short, foreign, tmp_path / "missing.lrn"):
        with pytest.raises(binding.LorannError) as e:
            binding.Index.from_file(p)
        assert e.value.code == -1


@pytest.mark.gpu
def test_library_reader(tmp_path):
    import torch
    from paper_2410_18926_amd import binding
    assert torch.cuda.is_available()
    rng = np.random.default_rng(8)
    for metric, with_P, with_ids in [(0, True, True), (1, False, False)]:
        ix = _index(rng, metric, with_P, with_ids)
        path = tmp_path / f"index{metric}.lrn"
        save_index(path, ix)
        q = rng.normal(size=(30, ix["d"])).astype(np.float32)
        a = binding.Index(**ix)
        f = binding.Index.from_file(path)
        a_ids, a_d = a.search(q, 5, 3, 40)
        f_ids, f_d = f.search(q, 5, 3, 40)
        np.testing.assert_array_equal(f_ids, a_ids)
        np.testing.assert_array_equal(f_d, a_d)
        o_ids, o_d = O.search(O.OracleIndex.from_file(path), q, 5, 3, 40)
        np.testing.assert_array_equal(f_ids, o_ids)
        a.close(); f.close()
