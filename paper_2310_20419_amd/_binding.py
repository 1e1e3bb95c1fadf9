"""ctypes marshalling for librnnd.so -- same names as the C entry points, no arithmetic."""
from __future__ import annotations

import ctypes
import os
import re

RNND_U8, RNND_F32, RNND_F16, RNND_BF16 = 0, 1, 2, 3
RNND_L2SQ = 0
RNND_MAX_R = 128
RNND_MAX_ROUNDS = 256

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = os.path.join(_HERE, "librnnd.so")
_HEADER = os.path.join(os.path.dirname(_HERE), "include", "rnnd.h")


class RnndError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("rnnd status %d: %s" % (status, message))
        self.status = status


class Stats(ctypes.Structure):
    _fields_ = [
        ("rounds", ctypes.c_int32),
        ("reverse_calls", ctypes.c_int32),
        ("kernel_variant", ctypes.c_int32),
        ("reserved", ctypes.c_int32),
        ("total_ms", ctypes.c_float),
        ("init_ms", ctypes.c_float),
        ("round_ms", ctypes.c_float * RNND_MAX_ROUNDS),
        ("scan_ms", ctypes.c_float * RNND_MAX_ROUNDS),
        ("reverse_ms", ctypes.c_float * RNND_MAX_ROUNDS),
        ("init_evals", ctypes.c_int64),
        ("active", ctypes.c_int64 * RNND_MAX_ROUNDS),
        ("proposals", ctypes.c_int64 * RNND_MAX_ROUNDS),
        ("algo_evals", ctypes.c_int64 * RNND_MAX_ROUNDS),
        ("exec_evals", ctypes.c_int64 * RNND_MAX_ROUNDS),
        ("gathered_rows", ctypes.c_int64 * RNND_MAX_ROUNDS),
        ("dropped", ctypes.c_int64 * RNND_MAX_ROUNDS),
    ]

    def as_dict(self) -> dict:
        n = min(self.rounds, RNND_MAX_ROUNDS)
        return {
            "rounds": self.rounds, "reverse_calls": self.reverse_calls,
            "kernel_variant": self.kernel_variant,
            "total_ms": self.total_ms, "init_ms": self.init_ms,
            "round_ms": list(self.round_ms[:n]), "scan_ms": list(self.scan_ms[:n]),
            "reverse_ms": list(self.reverse_ms[:max(0, self.reverse_calls)]),
            "init_evals": self.init_evals, "active": list(self.active[:n]),
            "proposals": list(self.proposals[:n]), "algo_evals": list(self.algo_evals[:n]),
            "exec_evals": list(self.exec_evals[:n]), "gathered_rows": list(self.gathered_rows[:n]),
            "dropped": list(self.dropped[:n]),
        }


def lib_path() -> str:
    return _LIB


def exported_symbols() -> list:
    """Function names include/rnnd.h declares."""
    text = open(_HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rnnd_[a-z_]+)\s*\(", text)))


_lib = None


def load_library():
    """Loads the in-tree librnnd.so; fails loudly if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            raise RnndError(-6, "librnnd.so is not built (run `python -m paper_2310_20419_amd.build`); "
                                "there is no CPU fallback")
        # PyTorch owns the device memory and streams handed to the library, so both must share one
        # HIP runtime: import torch first, so that librnnd.so binds to the runtime torch has loaded.
        import torch  # noqa: F401
        L = ctypes.CDLL(_LIB)
        c = ctypes
        vp, i64, i32, u64 = c.c_void_p, c.c_int64, c.c_int32, c.c_uint64
        L.rnnd_build.argtypes = [vp, i64, i32, c.c_int, c.c_int, i32, i32, i32, i32, u64, vp, vp, vp]
        L.rnnd_build_ex.argtypes = [vp, i64, i32, c.c_int, c.c_int, i32, i32, i32, i32, u64, vp, vp, vp,
                                    c.POINTER(Stats), vp]
        L.rnnd_build_wide.argtypes = [vp, i64, i32, c.c_int, c.c_int, i32, i32, i32, i32, i32, u64, vp, vp, vp,
                                      c.POINTER(Stats), vp]
        L.rnnd_build_blocks.argtypes = [vp, i64, i32, c.c_int, c.c_int, i32, i32, i32, i32, u64, i64, vp, vp, vp,
                                        c.POINTER(Stats), vp]
        L.rnnd_update_neighbors_blocks.argtypes = [vp, i64, i32, c.c_int, c.c_int, i32, vp, vp, i32, i64,
                                                   c.POINTER(Stats), vp]
        L.rnnd_workspace_bytes.argtypes = [i64, i32, c.c_int, i32, i64, c.POINTER(c.c_size_t)]
        L.rnnd_build_static.argtypes = L.rnnd_build.argtypes
        L.rnnd_release_workspace.argtypes = []
        L.rnnd_set_workspace_poison.argtypes = [c.c_int]
        L.rnnd_random_graph.argtypes = [vp, i64, i32, c.c_int, c.c_int, i32, i32, u64, vp, vp, vp]
        L.rnnd_update_neighbors.argtypes = [vp, i64, i32, c.c_int, c.c_int, i32, vp, vp, i32,
                                            c.POINTER(Stats), vp]
        L.rnnd_add_reverse_edges.argtypes = [i64, i32, vp, vp, vp]
        L.rnnd_add_reverse_edges_wide.argtypes = [i64, i32, i32, vp, vp, vp]
        L.rnnd_export_graph.argtypes = [i64, i32, vp, vp, vp, vp, vp]
        L.rnnd_search.argtypes = [vp, i64, i32, c.c_int, c.c_int, vp, vp, i32, vp, i64, i32, i32, i32, c.c_uint64,
                                  vp, vp, c.POINTER(c.c_int64), vp]
        L.rnnd_probe_gather.argtypes = [vp, i64, i64, i64, u64, c.POINTER(c.c_double), vp]
        L.rnnd_probe_gather_map.argtypes = [vp, i64, i64, i64, c.c_int, u64, c.POINTER(c.c_double), vp]
        L.rnnd_set_kernel_variant.argtypes = [c.c_int]
        L.rnnd_set_transpose_path.argtypes = [c.c_int]
        L.rnnd_set_scan_launches.argtypes = [c.c_int]
        L.rnnd_set_event_timing.argtypes = [c.c_int]
        L.rnnd_strerror.argtypes = [c.c_int]
        L.rnnd_strerror.restype = c.c_char_p
        L.rnnd_version.restype = c.c_int
        for name in ("rnnd_build", "rnnd_build_ex", "rnnd_workspace_bytes", "rnnd_random_graph",
                     "rnnd_update_neighbors", "rnnd_add_reverse_edges", "rnnd_export_graph", "rnnd_search",
                     "rnnd_set_kernel_variant", "rnnd_build_blocks", "rnnd_update_neighbors_blocks",
                     "rnnd_probe_gather", "rnnd_build_wide", "rnnd_build_static", "rnnd_release_workspace",
                     "rnnd_set_workspace_poison", "rnnd_add_reverse_edges_wide", "rnnd_set_transpose_path",
                     "rnnd_set_event_timing", "rnnd_probe_gather_map", "rnnd_set_scan_launches"):
            getattr(L, name).restype = c.c_int
        _lib = L
    return _lib


def rnnd_strerror(status: int) -> str:
    return load_library().rnnd_strerror(status).decode()


def rnnd_version() -> int:
    return load_library().rnnd_version()


def _check(rc: int):
    if rc != 0:
        raise RnndError(rc, rnnd_strerror(rc))


def _torch():
    import torch
    return torch


def _data_args(X):
    torch = _torch()
    if not (X.is_cuda and X.dim() == 2 and X.is_contiguous()):
        raise ValueError("X must be a contiguous 2-D tensor in device memory")
    if X.dtype == torch.uint8:
        dt = RNND_U8
    elif X.dtype == torch.float32:
        dt = RNND_F32
    elif X.dtype == torch.float16:
        dt = RNND_F16
    elif X.dtype == torch.bfloat16:
        dt = RNND_BF16
    else:
        raise ValueError("X must be uint8, float32, float16 or bfloat16")
    return X.data_ptr(), X.shape[0], X.shape[1], dt


def _stream(stream):
    torch = _torch()
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


RNND_STATIC_SCRATCH_BYTES = 64 << 20


def rnnd_workspace_bytes(N: int, d: int, dtype: int, R: int, rounds: int) -> int:
    b = ctypes.c_size_t(0)
    _check(load_library().rnnd_workspace_bytes(N, d, dtype, R, rounds, ctypes.byref(b)))
    return b.value


def rnnd_release_workspace():
    _check(load_library().rnnd_release_workspace())


def rnnd_set_workspace_poison(on: bool):
    _check(load_library().rnnd_set_workspace_poison(1 if on else 0))


def rnnd_set_event_timing(on: bool):
    """Per-round times of the statistics from HIP events (True) or from the device clock (False, the default)."""
    _check(load_library().rnnd_set_event_timing(1 if on else 0))


def rnnd_build_static(X, S: int, R: int, T1: int, T2: int, seed: int, graph, degree, metric: int = RNND_L2SQ,
                      stream=None):
    """rnnd_build_static: the caller passes the outputs (graph [N, R] int32, degree [N] int32, on X's device);
    nothing is allocated, here or in the library."""
    ptr, N, d, dt = _data_args(X)
    assert graph.is_cuda and graph.is_contiguous() and graph.shape == (N, R) and graph.element_size() == 4
    assert degree.is_cuda and degree.is_contiguous() and degree.shape == (N,) and degree.element_size() == 4
    _check(load_library().rnnd_build_static(ptr, N, d, dt, metric, S, R, T1, T2, seed, graph.data_ptr(),
                                            degree.data_ptr(), _stream(stream)))


def rnnd_build(X, S: int, R: int, T1: int, T2: int, seed: int, metric: int = RNND_L2SQ, stream=None):
    """rnnd_build: returns (graph [N, R] int32, -1 padded; degree [N] int32), both on X's device."""
    torch = _torch()
    ptr, N, d, dt = _data_args(X)
    graph = torch.empty((N, R), dtype=torch.int32, device=X.device)
    degree = torch.empty((N,), dtype=torch.int32, device=X.device)
    _check(load_library().rnnd_build(ptr, N, d, dt, metric, S, R, T1, T2, seed, graph.data_ptr(),
                                     degree.data_ptr(), _stream(stream)))
    return graph, degree


def rnnd_build_ex(X, S: int, R: int, T1: int, T2: int, seed: int, metric: int = RNND_L2SQ, stream=None,
                  want_keys: bool = True):
    """rnnd_build_ex: returns (graph, degree, keys [N, R] int64-typed uint64 or None, Stats)."""
    torch = _torch()
    ptr, N, d, dt = _data_args(X)
    graph = torch.empty((N, R), dtype=torch.int32, device=X.device)
    degree = torch.empty((N,), dtype=torch.int32, device=X.device)
    keys = torch.empty((N, R), dtype=torch.int64, device=X.device) if want_keys else None
    st = Stats()
    _check(load_library().rnnd_build_ex(ptr, N, d, dt, metric, S, R, T1, T2, seed, graph.data_ptr(),
                                        degree.data_ptr(), keys.data_ptr() if want_keys else None,
                                        ctypes.byref(st), _stream(stream)))
    return graph, degree, keys, st


def rnnd_build_wide(X, S: int, R: int, M: int, T1: int, T2: int, seed: int, metric: int = RNND_L2SQ, stream=None,
                    want_keys: bool = True):
    """rnnd_build_wide: returns (graph [N, M], degree, keys [N, M] int64-typed uint64 or None, Stats)."""
    torch = _torch()
    ptr, N, d, dt = _data_args(X)
    graph = torch.empty((N, M), dtype=torch.int32, device=X.device)
    degree = torch.empty((N,), dtype=torch.int32, device=X.device)
    keys = torch.empty((N, M), dtype=torch.int64, device=X.device) if want_keys else None
    st = Stats()
    _check(load_library().rnnd_build_wide(ptr, N, d, dt, metric, S, R, M, T1, T2, seed, graph.data_ptr(),
                                          degree.data_ptr(), keys.data_ptr() if want_keys else None,
                                          ctypes.byref(st), _stream(stream)))
    return graph, degree, keys, st


def rnnd_build_blocks(X, S: int, R: int, T1: int, T2: int, seed: int, blocks: int, metric: int = RNND_L2SQ,
                      stream=None, want_keys: bool = True):
    """rnnd_build_blocks: returns (graph, degree, keys [N, R] int64-typed uint64 or None, Stats)."""
    torch = _torch()
    ptr, N, d, dt = _data_args(X)
    graph = torch.empty((N, R), dtype=torch.int32, device=X.device)
    degree = torch.empty((N,), dtype=torch.int32, device=X.device)
    keys = torch.empty((N, R), dtype=torch.int64, device=X.device) if want_keys else None
    st = Stats()
    _check(load_library().rnnd_build_blocks(ptr, N, d, dt, metric, S, R, T1, T2, seed, blocks, graph.data_ptr(),
                                            degree.data_ptr(), keys.data_ptr() if want_keys else None,
                                            ctypes.byref(st), _stream(stream)))
    return graph, degree, keys, st


def rnnd_random_graph(X, S: int, R: int, seed: int, metric: int = RNND_L2SQ, stream=None):
    torch = _torch()
    ptr, N, d, dt = _data_args(X)
    keys = torch.empty((N, R), dtype=torch.int64, device=X.device)
    deg = torch.empty((N,), dtype=torch.int32, device=X.device)
    _check(load_library().rnnd_random_graph(ptr, N, d, dt, metric, S, R, seed, keys.data_ptr(),
                                            deg.data_ptr(), _stream(stream)))
    return keys, deg


def rnnd_update_neighbors(X, keys, deg, R: int, n_rounds: int = 1, metric: int = RNND_L2SQ, stream=None):
    """In place on (keys, deg); returns Stats."""
    ptr, N, d, dt = _data_args(X)
    assert keys.is_cuda and keys.is_contiguous() and keys.shape == (N, R) and keys.element_size() == 8
    assert deg.is_cuda and deg.is_contiguous() and deg.shape == (N,) and deg.element_size() == 4
    st = Stats()
    _check(load_library().rnnd_update_neighbors(ptr, N, d, dt, metric, R, keys.data_ptr(), deg.data_ptr(),
                                                n_rounds, ctypes.byref(st), _stream(stream)))
    return st


def rnnd_update_neighbors_blocks(X, keys, deg, R: int, blocks: int, n_passes: int = 1, metric: int = RNND_L2SQ,
                                 stream=None):
    """In place on (keys, deg); returns Stats."""
    ptr, N, d, dt = _data_args(X)
    assert keys.is_cuda and keys.is_contiguous() and keys.shape == (N, R) and keys.element_size() == 8
    assert deg.is_cuda and deg.is_contiguous() and deg.shape == (N,) and deg.element_size() == 4
    st = Stats()
    _check(load_library().rnnd_update_neighbors_blocks(ptr, N, d, dt, metric, R, keys.data_ptr(), deg.data_ptr(),
                                                       n_passes, blocks, ctypes.byref(st), _stream(stream)))
    return st


def rnnd_probe_gather(X, n_gather: int, seed: int = 1, stream=None) -> float:
    """GB/s of random whole-row gathers from X (measurement aid)."""
    assert X.is_cuda and X.is_contiguous() and X.dim() == 2
    out = ctypes.c_double(0.0)
    _check(load_library().rnnd_probe_gather(X.data_ptr(), X.shape[0], X.shape[1] * X.element_size(), n_gather, seed,
                                            ctypes.byref(out), _stream(stream)))
    return out.value


def rnnd_probe_gather_map(X, n_gather: int, lanes_per_row: int, seed: int = 1, stream=None) -> float:
    """GB/s of random whole-row gathers from X with lanes_per_row lanes reading a row together."""
    assert X.is_cuda and X.is_contiguous() and X.dim() == 2
    out = ctypes.c_double(0.0)
    _check(load_library().rnnd_probe_gather_map(X.data_ptr(), X.shape[0], X.shape[1] * X.element_size(), n_gather,
                                                lanes_per_row, seed, ctypes.byref(out), _stream(stream)))
    return out.value


def rnnd_add_reverse_edges(keys, deg, R: int, stream=None):
    N = keys.shape[0]
    assert keys.is_cuda and keys.is_contiguous() and keys.shape == (N, R) and keys.element_size() == 8
    assert deg.is_cuda and deg.is_contiguous() and deg.shape == (N,) and deg.element_size() == 4
    _check(load_library().rnnd_add_reverse_edges(N, R, keys.data_ptr(), deg.data_ptr(), _stream(stream)))


def rnnd_add_reverse_edges_wide(keys, deg, R: int, stream=None):
    """Rows are keys.shape[1] >= R slots wide."""
    N, M = keys.shape
    assert keys.is_cuda and keys.is_contiguous() and keys.element_size() == 8
    assert deg.is_cuda and deg.is_contiguous() and deg.shape == (N,) and deg.element_size() == 4
    _check(load_library().rnnd_add_reverse_edges_wide(N, R, M, keys.data_ptr(), deg.data_ptr(), _stream(stream)))


def rnnd_export_graph(keys, deg, R: int, stream=None):
    torch = _torch()
    N = keys.shape[0]
    graph = torch.empty((N, R), dtype=torch.int32, device=keys.device)
    degree = torch.empty((N,), dtype=torch.int32, device=keys.device)
    _check(load_library().rnnd_export_graph(N, R, keys.data_ptr(), deg.data_ptr(), graph.data_ptr(),
                                            degree.data_ptr(), _stream(stream)))
    return graph, degree


def rnnd_search(X, graph, degree, Q, L: int, K: int, k: int, seed: int, want_dist: bool = False,
                metric: int = RNND_L2SQ, stream=None):
    """Alg. 1 with the cap K on the GPU.  Returns (ids int32 [nq, k], dist_bits int32 [nq, k] or None, evals)."""
    torch = _torch()
    ptr, N, d, dt = _data_args(X)
    assert Q.is_cuda and Q.is_contiguous() and Q.dtype == X.dtype and Q.dim() == 2 and Q.shape[1] == d
    assert graph.is_cuda and graph.is_contiguous() and graph.dtype == torch.int32 and graph.shape[0] == N
    assert degree.is_cuda and degree.is_contiguous() and degree.dtype == torch.int32 and degree.shape == (N,)
    nq = Q.shape[0]
    ids = torch.empty((nq, k), dtype=torch.int32, device=X.device)
    dist = torch.empty((nq, k), dtype=torch.int32, device=X.device) if want_dist else None
    ev = ctypes.c_int64(0)
    _check(load_library().rnnd_search(ptr, N, d, dt, metric, graph.data_ptr(), degree.data_ptr(), graph.shape[1],
                                      Q.data_ptr(), nq, L, K, k, seed, ids.data_ptr(),
                                      dist.data_ptr() if want_dist else None, ctypes.byref(ev), _stream(stream)))
    return ids, dist, ev.value


def rnnd_set_transpose_path(path: int):
    _check(load_library().rnnd_set_transpose_path(path))


def rnnd_set_scan_launches(mode: int):
    _check(load_library().rnnd_set_scan_launches(mode))


def rnnd_set_kernel_variant(variant: int):
    _check(load_library().rnnd_set_kernel_variant(variant))


# ---- snapshot format helpers (host side, numpy): layout conversion only
def pack_keys(ids, dist_bits, flags, deg):
    """(ids int32 [N,R], dist_bits uint32 [N,R], flags uint8 [N,R], deg) -> uint64 keys [N,R]."""
    import numpy as np
    k = (dist_bits.astype(np.uint64) << np.uint64(32)) | \
        ((ids.astype(np.int64) & 0x7FFFFFFF).astype(np.uint64) << np.uint64(1)) | \
        (flags.astype(np.uint64) & np.uint64(1))
    pad = np.arange(ids.shape[1])[None, :] >= np.asarray(deg)[:, None]
    k[pad] = np.uint64(0xFFFFFFFFFFFFFFFF)
    return k


def unpack_keys(keys, deg):
    """uint64 keys [N,R] -> (ids int32 (-1 padded), dist_bits uint32, flags uint8)."""
    import numpy as np
    keys = keys.view(np.uint64) if keys.dtype != np.uint64 else keys
    ids = ((keys >> np.uint64(1)) & np.uint64(0x7FFFFFFF)).astype(np.int32)
    dist_bits = (keys >> np.uint64(32)).astype(np.uint32)
    flags = (keys & np.uint64(1)).astype(np.uint8)
    pad = np.arange(keys.shape[1])[None, :] >= np.asarray(deg)[:, None]
    ids[pad] = -1
    dist_bits[pad] = 0
    flags[pad] = 0
    return ids, dist_bits, flags
