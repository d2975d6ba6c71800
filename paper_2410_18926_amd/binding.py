"""Thin ctypes binding of the C-ABI library declared in include/lorann.h (argument marshalling only).

Every step of the search runs inside the HIP library.  Arrays may be torch tensors (CPU or GPU) or numpy
arrays; their memory is handed to the library as plain pointers.  Importing this module fails loudly when the
library has not been built (`python -m paper_2410_18926_amd.build`): there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
import pathlib

import numpy as np

try:
    import torch
except Exception:  # pragma: no cover - torch is part of the image
    torch = None

# (LORANN_LIB names another build of the same library: the host-sanitized one of build.build_sanitized)
LIB_PATH = pathlib.Path(os.environ.get("LORANN_LIB") or pathlib.Path(__file__).resolve().parent / "liblorann.so")

LORANN_IP, LORANN_L2, LORANN_COS = 0, 1, 2
LORANN_OK, LORANN_E_INVAL, LORANN_E_NOMEM, LORANN_E_DEVICE, LORANN_E_UNSUPPORTED = 0, -1, -2, -3, -4

EXPORTS = ["lorann_load_index", "lorann_load_index_file", "lorann_search", "lorann_search_async", "lorann_free_index", "lorann_last_error", "lorann_set_stream",
           "lorann_search_stages", "lorann_profile_enable", "lorann_profile_get", "lorann_set_exact_selection", "lorann_set_screen_mode",
           "lorann_profile_fallback_queries", "lorann_set_rerank", "lorann_set_column_scales", "lorann_set_first_rows", "lorann_search_lane", "lorann_lane_join", "lorann_set_gather_turns", "lorann_search_noalloc", "lorann_profile_gather_rows"]
NOALLOC_SCRATCH_BYTES = 32 << 20
LANES = 4
RERANK_F32, RERANK_F16, RERANK_NONE = 0, 1, 2
SCREEN_AUTO, SCREEN_MATRIX, SCREEN_DIGEST = 0, 1, 2


class LorannError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"lorann error {code}: {msg}")
        self.code = code


class _Stages(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("qproj", "q8", "dx", "sel", "z", "sigma", "cand_rows", "tau", "n_survivors", "y_off", "y", "rho0", "pmax")]


class _KernelTime(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("ms", C.c_double), ("launches", C.c_int64)]


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2410_18926_amd.build` "
                              "(there is no CPU or PyTorch fallback for the search)")
        L = C.CDLL(str(LIB_PATH))
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        L.lorann_load_index.restype = C.c_int
        L.lorann_load_index.argtypes = [C.POINTER(vp), i32, i64, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.lorann_search.restype = C.c_int
        L.lorann_search.argtypes = [vp, vp, i64, i32, i32, i32, vp, vp]
        L.lorann_search_async.restype = C.c_int
        L.lorann_search_async.argtypes = [vp, vp, i64, i32, i32, i32, vp, vp]
        L.lorann_search_noalloc.restype = C.c_int
        L.lorann_search_noalloc.argtypes = [vp, vp, i64, i32, i32, i32, vp, vp]
        L.lorann_search_stages.restype = C.c_int
        L.lorann_search_stages.argtypes = [vp, vp, i64, i32, i32, i32, vp, vp, C.POINTER(_Stages)]
        L.lorann_load_index_file.restype = C.c_int
        L.lorann_load_index_file.argtypes = [C.POINTER(C.c_void_p), C.c_char_p]
        L.lorann_free_index.restype = None
        L.lorann_free_index.argtypes = [vp]
        L.lorann_last_error.restype = C.c_char_p
        L.lorann_set_stream.restype = C.c_int
        L.lorann_set_stream.argtypes = [vp, vp]
        L.lorann_set_exact_selection.restype = C.c_int
        L.lorann_set_exact_selection.argtypes = [vp, i32]
        L.lorann_set_screen_mode.restype = C.c_int
        L.lorann_set_screen_mode.argtypes = [vp, i32]
        L.lorann_set_column_scales.restype = C.c_int
        L.lorann_set_column_scales.argtypes = [vp, vp, vp]
        L.lorann_set_first_rows.restype = C.c_int
        L.lorann_set_first_rows.argtypes = [vp, vp, vp]
        L.lorann_search_lane.restype = C.c_int
        L.lorann_search_lane.argtypes = [vp, i32, vp, i64, i32, i32, i32, vp, vp]
        L.lorann_set_gather_turns.restype = C.c_int
        L.lorann_set_gather_turns.argtypes = [vp, i32]
        L.lorann_lane_join.restype = C.c_int
        L.lorann_lane_join.argtypes = [vp, i32]
        L.lorann_set_rerank.restype = C.c_int
        L.lorann_set_rerank.argtypes = [vp, i32]
        L.lorann_profile_enable.restype = C.c_int
        L.lorann_profile_enable.argtypes = [vp, i32]
        L.lorann_profile_fallback_queries.restype = C.c_int64
        L.lorann_profile_fallback_queries.argtypes = [vp]
        L.lorann_profile_gather_rows.restype = C.c_int64
        L.lorann_profile_gather_rows.argtypes = [vp]
        L.lorann_profile_get.restype = C.c_int
        L.lorann_profile_get.argtypes = [vp, C.POINTER(_KernelTime), i32]
        _lib = L
    return _lib


def _check(rc: int):
    if rc != 0:
        raise LorannError(rc, lib().lorann_last_error().decode())


def _is_torch(a) -> bool:
    return torch is not None and isinstance(a, torch.Tensor)


def _prep(a, dtype_np, dtype_t):
    """Contiguous array of the right dtype (no device change); returns (keepalive, pointer)."""
    if a is None:
        return None, None
    if _is_torch(a):
        t = a.detach().to(dtype_t).contiguous()
        return t, t.data_ptr()
    n = np.ascontiguousarray(a, dtype=dtype_np)
    return n, n.ctypes.data


class Index:
    """A loaded index (owns device memory inside the library)."""

    def __init__(self, metric, n, d, dp, r, L, centroids, P, A, B, scale_A, scale_B, cluster_offsets, corpus, ids=None,
                 scale_A_columns=None, scale_B_points=None, first_row_A=None, first_row_B=None, **_):
        self._h = C.c_void_p()
        self.metric, self.n, self.d, self.dp, self.r, self.L = int(metric), int(n), int(d), int(dp), int(r), int(L)
        T = torch
        keep = [
            _prep(centroids, np.float32, T.float32 if T else None), _prep(P, np.float32, T.float32 if T else None),
            _prep(A, np.int8, T.int8 if T else None), _prep(B, np.int8, T.int8 if T else None),
            _prep(scale_A, np.float32, T.float32 if T else None), _prep(scale_B, np.float32, T.float32 if T else None),
            _prep(cluster_offsets, np.int64, T.int64 if T else None), _prep(corpus, np.float32, T.float32 if T else None),
            _prep(ids, np.int64, T.int64 if T else None),
        ]
        ptrs = [p for _, p in keep]
        _check(lib().lorann_load_index(C.byref(self._h), self.metric, self.n, self.d, self.dp, self.r, self.L, *ptrs))
        del keep
        if scale_A_columns is not None or scale_B_points is not None:
            self.set_column_scales(scale_A_columns, scale_B_points)
        if first_row_A is not None or first_row_B is not None:
            self.set_first_rows(first_row_A, first_row_B)

    @classmethod
    def from_arrays(cls, ix) -> "Index":
        """From a synth.IndexArrays or a dict with the same field names."""
        d = ix if isinstance(ix, dict) else {f: getattr(ix, f) for f in
                                             ("metric", "n", "d", "dp", "r", "L", "centroids", "P", "A", "B", "scale_A",
                                              "scale_B", "cluster_offsets", "corpus", "ids")}
        if not isinstance(ix, dict):
            d["scale_A_columns"] = getattr(ix, "scale_A_columns", None)
            d["scale_B_points"] = getattr(ix, "scale_B_points", None)
            d["first_row_A"] = getattr(ix, "first_row_A", None)
            d["first_row_B"] = getattr(ix, "first_row_B", None)
        return cls(**d)

    @classmethod
    def from_file(cls, path) -> "Index":
        """lorann_load_index_file: load a serialized index (see synth.index_file for the writer)."""
        self = cls.__new__(cls)
        self._h = C.c_void_p()
        _check(lib().lorann_load_index_file(C.byref(self._h), str(path).encode()))
        from .synth.index_file import read_header
        h = read_header(path)
        self.metric, self.n, self.d, self.dp, self.r, self.L = (int(h[k]) for k in ("metric", "n", "d", "dp", "r", "L"))
        return self

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            lib().lorann_free_index(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_stream(self, stream_handle: int | None):
        _check(lib().lorann_set_stream(self._h, C.c_void_p(stream_handle or 0)))

    def use_torch_stream(self):
        """Run on torch's current stream of the current device."""
        self.set_stream(torch.cuda.current_stream().cuda_stream)

    def _outputs(self, queries, nq, k):
        if _is_torch(queries):
            ids = torch.empty((nq, k), dtype=torch.int64, device=queries.device)
            dists = torch.empty((nq, k), dtype=torch.float32, device=queries.device)
            return ids, dists, ids.data_ptr(), dists.data_ptr()
        ids, dists = np.empty((nq, k), np.int64), np.empty((nq, k), np.float32)
        return ids, dists, ids.ctypes.data, dists.ctypes.data

    def search(self, queries, k: int, w: int, m: int, out=None, asynchronous: bool = False, lane: int | None = None):
        """lorann_search: returns (ids [nq,k] int64, dists [nq,k] float32) of the same kind as `queries`.
        asynchronous=True (device tensors only) calls lorann_search_async: the results are complete once the
        index's stream has been synchronised.  lane=i calls lorann_search_lane (enqueue only, on lane i of the
        index); the results are complete on the index's stream after lane_join(i)."""
        if asynchronous or lane is not None:
            # the call returns before the kernels have read the queries: a converted temporary would be released (and
            # its memory handed out again) while a library-owned stream may still read it
            # (host arrays are passed on as they are: the library refuses them)
            if _is_torch(queries) and queries.is_cuda and not (queries.dtype == torch.float32 and queries.is_contiguous()):
                raise ValueError("asynchronous / lane searches need a contiguous float32 device tensor (no copy is made)")
        qk, qptr = _prep(queries, np.float32, torch.float32 if torch else None)
        nq = int(qk.shape[0])
        if qk.ndim != 2 or int(qk.shape[1]) != self.d:
            raise ValueError(f"queries must be [nq, {self.d}]")
        if out is None:
            ids, dists, ip, dptr = self._outputs(qk, nq, k)
        else:
            ids, dists = out
            ip, dptr = (ids.data_ptr(), dists.data_ptr()) if _is_torch(ids) else (ids.ctypes.data, dists.ctypes.data)
        if lane is not None:
            _check(lib().lorann_search_lane(self._h, int(lane), qptr, nq, k, w, m, ip, dptr))
        else:
            _check((lib().lorann_search_async if asynchronous else lib().lorann_search)(self._h, qptr, nq, k, w, m, ip, dptr))
        return ids, dists

    def search_noalloc(self, queries, k: int, w: int, m: int, out):
        """lorann_search_noalloc: enqueue only, nothing is allocated (not here either: the caller passes contiguous
        float32 device queries and the two output tensors)."""
        ids, dists = out
        if not (_is_torch(queries) and queries.is_cuda and queries.dtype == torch.float32 and queries.is_contiguous()):
            raise ValueError("search_noalloc needs a contiguous float32 device tensor")
        if queries.ndim != 2 or int(queries.shape[1]) != self.d:
            raise ValueError(f"queries must be [nq, {self.d}]")
        _check(lib().lorann_search_noalloc(self._h, queries.data_ptr(), int(queries.shape[0]), k, w, m, ids.data_ptr(), dists.data_ptr()))
        return ids, dists

    def set_gather_turns(self, on: bool):
        _check(lib().lorann_set_gather_turns(self._h, 1 if on else 0))

    def lane_join(self, lane: int):
        _check(lib().lorann_lane_join(self._h, int(lane)))

    def search_stages(self, queries, k: int, w: int, m: int, y_off=None):
        """lorann_search_stages with host outputs: (ids, dists, dict of numpy arrays)."""
        qk, qptr = _prep(queries, np.float32, torch.float32 if torch else None)
        nq = int(qk.shape[0])
        ids, dists = np.empty((nq, k), np.int64), np.empty((nq, k), np.float32)
        st = dict(qproj=np.zeros((nq, self.dp), np.float32), q8=np.zeros((nq, self.dp), np.int8),
                  dx=np.zeros(nq, np.float32), sel=np.zeros((nq, w), np.int32), z=np.zeros((nq, w, self.r), np.int8),
                  sigma=np.zeros((nq, w), np.float32), cand_rows=np.zeros((nq, m), np.int32),
                  tau=np.zeros(nq, np.float32), n_survivors=np.zeros(nq, np.int32), rho0=np.zeros((nq, w), np.float32),
                  pmax=np.full((nq, w), np.nan, np.float32))
        cs = _Stages()
        for name in st:
            setattr(cs, name, st[name].ctypes.data)
        if y_off is not None:
            y_off = np.ascontiguousarray(y_off, np.int64)
            assert y_off.shape == (nq * w + 1,)
            st["y"] = np.zeros(int(y_off[-1]), np.int32)
            cs.y_off, cs.y = y_off.ctypes.data, st["y"].ctypes.data
        _check(lib().lorann_search_stages(self._h, qptr, nq, k, w, m, ids.ctypes.data, dists.ctypes.data, C.byref(cs)))
        return ids, dists, st

    def set_exact_selection(self, on: bool):
        _check(lib().lorann_set_exact_selection(self._h, 1 if on else 0))

    def set_screen_mode(self, mode: int):
        _check(lib().lorann_set_screen_mode(self._h, int(mode)))

    def set_column_scales(self, scale_A_columns, scale_B_points):
        """One step size per column of A_c ([L, r]) and per corpus row ([n]) instead of one per cluster; None, None
        goes back to the per-cluster step sizes given at load time."""
        T = torch
        ka, pa = _prep(scale_A_columns, np.float32, T.float32 if T else None)
        kb, pb = _prep(scale_B_points, np.float32, T.float32 if T else None)
        _check(lib().lorann_set_column_scales(self._h, pa, pb))

    def set_first_rows(self, first_row_A, first_row_B):
        """Mixed-precision decomposition: the unquantized first row of every A_c ([L, r]) and B_c ([n], one value per
        corpus row); needs the column step sizes.  None, None switches it off."""
        T = torch
        ka, pa = _prep(first_row_A, np.float32, T.float32 if T else None)
        kb, pb = _prep(first_row_B, np.float32, T.float32 if T else None)
        _check(lib().lorann_set_first_rows(self._h, pa, pb))

    def set_rerank(self, mode: int):
        """RERANK_F32 (default), RERANK_F16 (half-precision copy of the corpus) or RERANK_NONE (no re-ranking step)."""
        _check(lib().lorann_set_rerank(self._h, int(mode)))

    def profile_enable(self, on=True):
        """True / 1: every kernel; 2: only the re-rank gather kernel; False / 0: off."""
        _check(lib().lorann_profile_enable(self._h, int(on)))

    def profile_fallback_queries(self) -> int:
        return int(lib().lorann_profile_fallback_queries(self._h))

    def profile_gather_rows(self) -> int:
        """Rows the grouped re-rank of the latest lane-0 batch fetched (-1: it did not run)."""
        return int(lib().lorann_profile_gather_rows(self._h))

    def profile_get(self) -> dict:
        """{kernel name: (total ms, launches)} since profiling was enabled."""
        n = lib().lorann_profile_get(self._h, None, 0)
        if n < 0:
            _check(n)
        arr = (_KernelTime * n)()
        lib().lorann_profile_get(self._h, arr, n)
        return {a.name.decode(): (a.ms, a.launches) for a in arr}
