"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every declared symbol, and
rejects invalid arguments before touching the device."""
import ctypes as C
import pathlib
import re

import numpy as np
import pytest

ROOT = pathlib.Path(__file__).resolve().parent.parent


@pytest.fixture(scope="module")
def B():
    from paper_2410_18926_amd import build, binding
    if not binding.LIB_PATH.exists():
        build.build()
    return binding


def test_library_exports_every_declared_symbol(B):
    header = (ROOT / "include" / "lorann.h").read_text()
    declared = set(re.findall(r"\b(lorann_[a-z_]+)\s*\(", header))
    declared -= {"lorann_index"}
    assert declared == set(B.EXPORTS)
    lib = B.lib()
    for name in declared:
        assert getattr(lib, name) is not None


def test_header_enums_match_binding(B):
    header = (ROOT / "include" / "lorann.h").read_text()
    for name, val in (("LORANN_IP", 0), ("LORANN_L2", 1), ("LORANN_COS", 2), ("LORANN_OK", 0), ("LORANN_E_INVAL", -1),
                      ("LORANN_E_NOMEM", -2), ("LORANN_E_DEVICE", -3), ("LORANN_E_UNSUPPORTED", -4)):
        assert re.search(rf"{name}\s*=\s*{val}\b", header), name
        assert getattr(B, name) == val


def _args(n=10, d=16, dp=16, r=8, L=2):
    return dict(metric=0, n=n, d=d, dp=dp, r=r, L=L, centroids=np.zeros((L, dp), np.float32), P=None,
                A=np.zeros((L, r, dp), np.int8), B=np.zeros((n, r), np.int8), scale_A=np.ones(L, np.float32),
                scale_B=np.ones(L, np.float32), cluster_offsets=np.array([0, 4, n], np.int64),
                corpus=np.zeros((n, d), np.float32), ids=None)


@pytest.mark.parametrize("change,code", [
    (dict(metric=7), -1),
    (dict(n=0), -1),
    (dict(dp=8, d=16), -1),                                   # P = NULL needs dp == d
    (dict(dp=24, d=24), -1),                                  # dp not a multiple of 16
    (dict(r=12), -1),                                         # r not a multiple of 8
    (dict(r=72), -4),                                         # beyond LORANN_MAX_R
    (dict(dp=2048, d=2048), -4),                              # beyond LORANN_MAX_DP
    (dict(cluster_offsets=np.array([0, 6, 4], np.int64)), -1),    # does not end at n
    (dict(cluster_offsets=np.array([1, 4, 10], np.int64)), -1),   # does not start at 0
    (dict(cluster_offsets=np.array([0, 12, 10], np.int64)), -1),  # decreasing
    (dict(corpus=None), -1),
])
def test_load_rejects_invalid_arguments_without_a_device(B, change, code):
    a = _args()
    a.update(change)
    for key in ("centroids", "A", "B", "corpus"):             # keep shapes consistent with changed sizes
        pass
    with pytest.raises(B.LorannError) as e:
        B.Index(**a)
    assert e.value.code == code
    assert str(e.value)


def test_search_on_null_index_is_rejected(B):
    lib = B.lib()
    rc = lib.lorann_search(None, None, 1, 1, 1, 1, None, None)
    assert rc == -1 and b"NULL" in lib.lorann_last_error()
    lib.lorann_free_index(None)                                # documented no-op


def test_every_entry_point_rejects_a_null_index(B):
    lib = B.lib()
    calls = [lambda: lib.lorann_search_async(None, None, 1, 1, 1, 1, None, None),
             lambda: lib.lorann_search_lane(None, 0, None, 1, 1, 1, 1, None, None),
             lambda: lib.lorann_lane_join(None, 0),
             lambda: lib.lorann_set_gather_turns(None, 1),
             lambda: lib.lorann_set_rerank(None, 0),
             lambda: lib.lorann_set_column_scales(None, None, None),
             lambda: lib.lorann_set_first_rows(None, None, None),
             lambda: lib.lorann_set_exact_selection(None, 1),
             lambda: lib.lorann_set_screen_mode(None, 0),
             lambda: lib.lorann_search_noalloc(None, None, 1, 1, 1, 1, None, None),
             lambda: lib.lorann_set_stream(None, None),
             lambda: lib.lorann_profile_enable(None, 1)]
    for call in calls:
        assert call() == B.LORANN_E_INVAL
        assert b"NULL" in lib.lorann_last_error()
    assert lib.lorann_profile_fallback_queries(None) == -1
    assert lib.lorann_profile_gather_rows(None) == -1


def test_header_constants_match_binding(B):
    header = (ROOT / "include" / "lorann.h").read_text()
    assert int(re.search(r"#define LORANN_LANES (\d+)", header).group(1)) == B.LANES
    for name, val in (("LORANN_RERANK_F32", B.RERANK_F32), ("LORANN_RERANK_F16", B.RERANK_F16), ("LORANN_RERANK_NONE", B.RERANK_NONE),
                      ("LORANN_SCREEN_AUTO", B.SCREEN_AUTO), ("LORANN_SCREEN_MATRIX", B.SCREEN_MATRIX), ("LORANN_SCREEN_DIGEST", B.SCREEN_DIGEST)):
        assert re.search(rf"{name}\s*=\s*{val}\b", header), name


def test_bench_refuses_more_than_one_gpu_and_a_missing_gpu():
    """bench.py measures one GPU: --gpus 2 exits with a message before anything is imported; without a GPU it says
    that no CPU fallback exists (this test runs where there is none)."""
    import subprocess, sys
    r = subprocess.run([sys.executable, str(ROOT / "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
    import torch
    if not torch.cuda.is_available():
        r = subprocess.run([sys.executable, str(ROOT / "bench.py")], capture_output=True, text=True, timeout=300)
        assert r.returncode == 2 and "needs the GPU" in r.stderr and r.stdout.strip() == ""
