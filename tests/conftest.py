import pathlib
import sys

import pytest

ROOT = pathlib.Path(__file__).resolve().parent.parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run on the GPU box)")


@pytest.fixture(scope="session")
def small_workloads():
    """Small synthetic workloads (seconds on CPU) covering the three metrics, with and without projection."""
    from paper_2410_18926_amd.synth.workloads import Workload, IP, L2, COS
    return {
        "l2_noP": Workload("t-l2", 91, n=3000, d=32, nq=40, G=12, alpha=None, normalize=False, lognormal_norms=None,
                           metric=L2, L=12, dp=32, r=8, w=4, m=50, n_train=1500, w_train=4),
        "ip_P": Workload("t-ip", 92, n=3000, d=48, nq=40, G=12, alpha=1.0, normalize=True, lognormal_norms=None,
                         metric=IP, L=10, dp=16, r=8, w=3, m=40, n_train=1500, w_train=3),
        "cos_P": Workload("t-cos", 93, n=2500, d=40, nq=40, G=10, alpha=0.8, normalize=True, lognormal_norms=None,
                          metric=COS, L=9, dp=32, r=16, w=3, m=30, n_train=1200, w_train=3),
        "l2_P_norms": Workload("t-l2n", 94, n=2500, d=40, nq=40, G=10, alpha=1.0, normalize=True,
                               lognormal_norms=0.5, metric=L2, L=9, dp=16, r=8, w=4, m=60, n_train=1200, w_train=4),
    }


@pytest.fixture(scope="session")
def small_indexes(small_workloads):
    from paper_2410_18926_amd.synth import make_dataset, build_index
    out = {}
    for name, wl in small_workloads.items():
        corpus, queries = make_dataset(wl)
        ix = build_index(corpus, wl, keep_float=True)
        out[name] = (wl, ix, corpus.numpy(), queries.numpy())
    return out


@pytest.fixture(scope="session")
def small_indexes_columns(small_workloads):
    """The same workloads quantized with one step size per column of A_c and of B_c (Sec. 3.3 as printed)."""
    from paper_2410_18926_amd.synth import make_dataset, build_index
    out = {}
    for name, wl in small_workloads.items():
        corpus, queries = make_dataset(wl)
        ix = build_index(corpus, wl, keep_float=True, column_scales=True)
        out[name] = (wl, ix, corpus.numpy(), queries.numpy())
    return out


@pytest.fixture(scope="session")
def small_indexes_mixed(small_workloads):
    """The same workloads with the first row of every A_c and B_c kept in float (Sec. 4.2 mixed precision)."""
    from paper_2410_18926_amd.synth import make_dataset, build_index
    out = {}
    for name, wl in small_workloads.items():
        corpus, queries = make_dataset(wl)
        ix = build_index(corpus, wl, keep_float=True, mixed_precision=True)
        out[name] = (wl, ix, corpus.numpy(), queries.numpy())
    return out
