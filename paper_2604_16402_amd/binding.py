"""Thin ctypes binding over libgrab.so: same names as the C ABI in include/grab.h, argument
marshalling only.  torch tensors (device or CPU) and numpy arrays are passed as raw
pointers; every step of the path runs inside the library's HIP kernels.  There is no
fallback: without the built library, or without a GPU, calls raise.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libgrab.so")

OK, EINVAL, ESTATE, EFULL, ENOMEM, EHIP = range(6)
STATUS_NAMES = {OK: "GRAB_OK", EINVAL: "GRAB_EINVAL", ESTATE: "GRAB_ESTATE", EFULL: "GRAB_EFULL",
                ENOMEM: "GRAB_ENOMEM", EHIP: "GRAB_EHIP"}
L2SQ, IP = 0, 1
P_SEARCH_WIDTH, P_MAX_ITER, P_N_SEEDS, P_VISITED_CAP, P_SEED_SALT, P_ALPHA, P_APPEND_BEAM, P_PROFILE, P_REMOTE_MODE, \
    P_N_PROXIMAL, P_REMOTE_WINDOW, P_APPEND_REMOTE_CANDS = range(12)
PARAMS = dict(search_width=P_SEARCH_WIDTH, max_iter=P_MAX_ITER, n_seeds=P_N_SEEDS, visited_cap=P_VISITED_CAP,
              seed_salt=P_SEED_SALT, alpha=P_ALPHA, append_beam=P_APPEND_BEAM, profile=P_PROFILE,
              remote_mode=P_REMOTE_MODE, n_proximal=P_N_PROXIMAL, remote_window=P_REMOTE_WINDOW,
              append_remote_cands=P_APPEND_REMOTE_CANDS)
EMPTY = 0xFFFFFFFF

EXPORTS = ["grab_create", "grab_destroy", "grab_last_error", "grab_build_buckets", "grab_load_graph",
           "grab_build_graph", "grab_build_remote", "grab_search_range", "grab_search_range_noalloc", "grab_append_batch", "grab_set_param", "grab_get_sizes", "grab_get_layout",
           "grab_get_graph", "grab_get_rows", "grab_select_range", "grab_get_counters", "grab_get_timing", "grab_get_append_stats",
           "grab_probe_gather", "grab_attr_image", "grab_attr_value", "grab_build_buckets_f32", "grab_search_range_f32",
           "grab_append_batch_f32"]

_lib = None


class GrabError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


def load_library() -> ctypes.CDLL:
    """dlopen the in-tree libgrab.so and declare its signatures.  Raises if it is not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_2604_16402_amd.build` "
                           "(or __graft_entry__.build()) first")
    # torch ships its own copy of the HIP runtime; load it first so that this library, torch's
    # allocator and torch's streams all live in one runtime (device pointers are shared)
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.grab_create.argtypes = [ctypes.POINTER(vp), i32, i32, vp]
    lib.grab_destroy.argtypes = [vp]
    lib.grab_destroy.restype = None
    lib.grab_last_error.argtypes = [vp]
    lib.grab_last_error.restype = ctypes.c_char_p
    lib.grab_build_buckets.argtypes = [vp, vp, vp, i64, i32, i64]
    lib.grab_load_graph.argtypes = [vp, vp, i32, vp, i32]
    lib.grab_build_graph.argtypes = [vp, i32, i32, i32]
    lib.grab_build_remote.argtypes = [vp]
    lib.grab_search_range.argtypes = [vp, vp, vp, vp, i64, i32, i32, vp, vp]
    lib.grab_search_range_noalloc.argtypes = [vp, vp, vp, vp, i64, i32, i32, vp, vp]
    lib.grab_append_batch.argtypes = [vp, vp, vp, i64]
    lib.grab_set_param.argtypes = [vp, i32, ctypes.c_double]
    lib.grab_get_sizes.argtypes = [vp, vp]
    lib.grab_get_layout.argtypes = [vp, vp, vp, vp]
    lib.grab_get_graph.argtypes = [vp, vp]
    lib.grab_get_rows.argtypes = [vp, vp, vp]
    lib.grab_select_range.argtypes = [vp, vp, vp, i64, i32, vp, vp]
    lib.grab_get_counters.argtypes = [vp, vp, i64]
    lib.grab_get_timing.argtypes = [vp, vp]
    lib.grab_get_append_stats.argtypes = [vp, vp, vp]
    lib.grab_probe_gather.argtypes = [vp, i64, i32, vp, vp]
    lib.grab_attr_image.argtypes = [ctypes.c_float]
    lib.grab_attr_value.argtypes = [i32]
    lib.grab_build_buckets_f32.argtypes = [vp, vp, vp, i64, i32, i64]
    lib.grab_search_range_f32.argtypes = [vp, vp, vp, vp, i64, i32, i32, vp, vp]
    lib.grab_append_batch_f32.argtypes = [vp, vp, vp, i64]
    for name in EXPORTS:
        if name not in ("grab_destroy", "grab_last_error", "grab_attr_image", "grab_attr_value"):
            getattr(lib, name).restype = ctypes.c_int
    lib.grab_attr_image.restype = i32
    lib.grab_attr_value.restype = ctypes.c_float
    _lib = lib
    return lib


def attr_image(x: float) -> int:
    """Order-preserving int32 image the library stores for a float attribute."""
    return int(load_library().grab_attr_image(ctypes.c_float(x)))


def attr_value(image: int) -> float:
    return float(load_library().grab_attr_value(int(image)))


def _ptr(x, dtype, count: Optional[int] = None):
    """Raw address of a contiguous torch tensor or numpy array of the given dtype."""
    if x is None:
        return None
    if isinstance(x, np.ndarray):
        if x.dtype != np.dtype(dtype) or not x.flags["C_CONTIGUOUS"]:
            raise TypeError(f"expected contiguous {np.dtype(dtype)} array, got {x.dtype}")
        if count is not None and x.size < count:
            raise ValueError("buffer too small")
        return x.ctypes.data
    import torch
    if isinstance(x, torch.Tensor):
        want = {np.dtype(np.float32): torch.float32, np.dtype(np.int32): torch.int32,
                np.dtype(np.uint32): (torch.uint32, torch.int32), np.dtype(np.int64): torch.int64}[np.dtype(dtype)]
        ok = x.dtype in want if isinstance(want, tuple) else x.dtype == want
        if not ok or not x.is_contiguous():
            raise TypeError(f"expected contiguous {dtype} tensor, got {x.dtype}")
        if count is not None and x.numel() < count:
            raise ValueError("buffer too small")
        return x.data_ptr()
    raise TypeError(type(x))


class Index:
    """One ``grab_index`` handle.  Methods mirror the C calls one to one."""

    def __init__(self, dim: int, metric: int = L2SQ, stream: Optional[int] = None):
        self._lib = load_library()
        self._h = ctypes.c_void_p()
        st = self._lib.grab_create(ctypes.byref(self._h), dim, metric, ctypes.c_void_p(stream or 0))
        if st != OK:
            raise GrabError(st, "grab_create rejected its arguments")
        self.dim, self.metric = dim, metric
        self._params = {}

    def _check(self, st: int):
        if st != OK:
            raise GrabError(st, self._lib.grab_last_error(self._h).decode())

    def close(self):
        if self._h:
            self._lib.grab_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_param(self, name: str, value: float):
        self._check(self._lib.grab_set_param(self._h, PARAMS[name], float(value)))
        self._params[name] = value

    def build_buckets(self, vectors, attrs, n_buckets: int, n_cap: Optional[int] = None):
        n = int(vectors.shape[0])
        if int(vectors.shape[1]) != self.dim:
            raise ValueError("vector dimension does not match the index")
        self._check(self._lib.grab_build_buckets(self._h, _ptr(vectors, np.float32, n * self.dim),
                                                 _ptr(attrs, np.int32, n), n, n_buckets, n if n_cap is None else n_cap))

    def build_buckets_f32(self, vectors, attrs, n_buckets: int, n_cap: Optional[int] = None):
        n = int(vectors.shape[0])
        if int(vectors.shape[1]) != self.dim:
            raise ValueError("vector dimension does not match the index")
        self._check(self._lib.grab_build_buckets_f32(self._h, _ptr(vectors, np.float32, n * self.dim),
                                                     _ptr(attrs, np.float32, n), n, n_buckets, n if n_cap is None else n_cap))

    def load_graph(self, local_adj, remote_adj):
        n = self.sizes()["n"]
        kl = int(local_adj.shape[1]) if local_adj is not None else 0
        kr = int(remote_adj.shape[1]) if remote_adj is not None else 0
        if (kl and int(local_adj.shape[0]) != n) or (kr and int(remote_adj.shape[0]) != n):
            raise ValueError("adjacency must have one row per object in the index")
        self._check(self._lib.grab_load_graph(self._h, _ptr(local_adj, np.uint32, n * kl) if kl else None, kl,
                                              _ptr(remote_adj, np.uint32, n * kr) if kr else None, kr))

    def build_graph(self, k_local: int, k_remote: int, pool: int = 0):
        self._check(self._lib.grab_build_graph(self._h, k_local, k_remote, pool))

    def build_remote(self):
        self._check(self._lib.grab_build_remote(self._h))

    def search_range(self, queries, lo, hi, k: int, beam: int, out_ids=None, out_dist=None):
        """Returns (ids[nq,k], dist[nq,k]); outputs are numpy unless device tensors are passed in."""
        nq = int(queries.shape[0])
        if out_ids is None:
            out_ids = np.empty((nq, k), dtype=np.uint32)
        if out_dist is None:
            out_dist = np.empty((nq, k), dtype=np.float32)
        self._check(self._lib.grab_search_range(self._h, _ptr(queries, np.float32, nq * self.dim),
                                                _ptr(lo, np.int32, nq), _ptr(hi, np.int32, nq), nq, k, beam,
                                                _ptr(out_ids, np.uint32, nq * k), _ptr(out_dist, np.float32, nq * k)))
        return out_ids, out_dist

    def search_range_noalloc(self, queries, lo, hi, k: int, beam: int, out_ids, out_dist):
        """search_range without any allocation inside the library: device tensors only."""
        nq = int(queries.shape[0])
        self._check(self._lib.grab_search_range_noalloc(self._h, _ptr(queries, np.float32, nq * self.dim),
                                                        _ptr(lo, np.int32, nq), _ptr(hi, np.int32, nq), nq, k, beam,
                                                        _ptr(out_ids, np.uint32, nq * k), _ptr(out_dist, np.float32, nq * k)))
        return out_ids, out_dist

    def search_range_f32(self, queries, lo, hi, k: int, beam: int, out_ids=None, out_dist=None):
        """search_range with fp32 range bounds."""
        nq = int(queries.shape[0])
        if out_ids is None:
            out_ids = np.empty((nq, k), dtype=np.uint32)
        if out_dist is None:
            out_dist = np.empty((nq, k), dtype=np.float32)
        self._check(self._lib.grab_search_range_f32(self._h, _ptr(queries, np.float32, nq * self.dim),
                                                    _ptr(lo, np.float32, nq), _ptr(hi, np.float32, nq), nq, k, beam,
                                                    _ptr(out_ids, np.uint32, nq * k), _ptr(out_dist, np.float32, nq * k)))
        return out_ids, out_dist

    def append_batch_f32(self, vectors, attrs):
        m = int(vectors.shape[0])
        self._check(self._lib.grab_append_batch_f32(self._h, _ptr(vectors, np.float32, m * self.dim),
                                                    _ptr(attrs, np.float32, m), m))

    def append_batch(self, vectors, attrs):
        m = int(vectors.shape[0])
        self._check(self._lib.grab_append_batch(self._h, _ptr(vectors, np.float32, m * self.dim),
                                                _ptr(attrs, np.int32, m), m))

    def sizes(self) -> dict:
        out = np.zeros(8, dtype=np.int64)
        self._check(self._lib.grab_get_sizes(self._h, out.ctypes.data))
        return dict(zip(["n", "n_slots", "n_buckets", "k_local", "k_remote", "dim", "metric", "has_graph"], out.tolist()))

    def get_layout(self):
        s = self.sizes()
        table = np.empty((s["n_buckets"], 6), dtype=np.int32)
        id2slot = np.empty(s["n"], dtype=np.uint32)
        slot2id = np.empty(s["n_slots"], dtype=np.uint32)
        self._check(self._lib.grab_get_layout(self._h, table.ctypes.data, id2slot.ctypes.data, slot2id.ctypes.data))
        return table, id2slot, slot2id

    def get_graph(self) -> np.ndarray:
        s = self.sizes()
        adj = np.empty((s["n_slots"], s["k_local"] + s["k_remote"]), dtype=np.uint32)
        self._check(self._lib.grab_get_graph(self._h, adj.ctypes.data))
        return adj

    def get_rows(self):
        s = self.sizes()
        x = np.empty((s["n_slots"], s["dim"]), dtype=np.float32)
        a = np.empty(s["n_slots"], dtype=np.int32)
        self._check(self._lib.grab_get_rows(self._h, x.ctypes.data, a.ctypes.data))
        return x, a

    def select_range(self, lo, hi, beam: int = 64):
        nq = int(lo.shape[0])
        info = np.empty((nq, 6), dtype=np.int32)
        S = int(self._params.get("n_seeds", 0)) or min(beam, 64)
        seeds = np.empty((nq, S), dtype=np.uint32)
        self._check(self._lib.grab_select_range(self._h, _ptr(lo, np.int32, nq), _ptr(hi, np.int32, nq), nq, beam,
                                                info.ctypes.data, seeds.ctypes.data))
        return info, seeds

    def get_counters(self, nq: int) -> np.ndarray:
        out = np.empty((nq, 8), dtype=np.uint32)
        self._check(self._lib.grab_get_counters(self._h, out.ctypes.data, nq))
        return out

    def probe_gather(self, waves: int = 65536, batches: int = 40):
        """(ms, bytes) of a launch that only reads random vector rows of the index."""
        ms = np.zeros(1, dtype=np.float32)
        nbytes = np.zeros(1, dtype=np.float64)
        self._check(self._lib.grab_probe_gather(self._h, waves, batches, ms.ctypes.data, nbytes.ctypes.data))
        return float(ms[0]), float(nbytes[0])

    APPEND_STATS = ["requests_local", "requests_remote", "groups_local", "groups_remote", "applied_local", "applied_remote",
                    "candidates_scanned", "remote_rows_evaluated", "local_requests_passed", "search_evals", "search_parents"]

    def get_append_stats(self, timing: bool = False):
        """Work counters of the last append_batch as a dict; with timing=True also `ms` = (search,
        forward selection, new rows + sorting, rewiring); needs set_param("profile", 1)."""
        counts = np.zeros(12, dtype=np.uint64)
        ms = np.zeros(4, dtype=np.float32)
        self._check(self._lib.grab_get_append_stats(self._h, counts.ctypes.data, ms.ctypes.data if timing else None))
        out = dict(zip(self.APPEND_STATS, (int(x) for x in counts)))
        if timing:
            out["ms"] = [float(x) for x in ms]
        return out

    def get_timing(self):
        """(select_ms, beam_ms) of the last search; needs set_param("profile", 1) before it."""
        out = np.zeros(2, dtype=np.float32)
        self._check(self._lib.grab_get_timing(self._h, out.ctypes.data))
        return float(out[0]), float(out[1])
