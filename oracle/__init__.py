"""CPU oracle for the RNN-Descent construction rounds -- TEST INFRASTRUCTURE.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  The product package never does, and this
package never imports the product.

The arithmetic lives in ``rnnd_oracle.c`` (plain single-threaded C, written from
the paper's Alg. 1, 3, 4, 5, 6 and Eq. 2-4); this module only compiles it with
gcc and marshals numpy arrays through ctypes.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rnnd_oracle.c")
_LIB = os.path.join(_HERE, "librnnd_oracle.so")

U8, F32 = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-ffp-contract=off", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.orc_mix64.restype = ctypes.c_uint64
        L.orc_mix64.argtypes = [ctypes.c_uint64]
        L.orc_draw.restype = ctypes.c_uint64
        L.orc_draw.argtypes = [ctypes.c_uint64] * 3
        L.orc_delta.restype = ctypes.c_double
        _lib = L
    return _lib


def _dt(X: np.ndarray) -> int:
    if X.dtype == np.uint8:
        return U8
    if X.dtype == np.float32:
        return F32
    raise TypeError("oracle takes uint8 or float32 data, got %s" % X.dtype)


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _chk(X):
    assert X.ndim == 2 and X.flags.c_contiguous
    return X


@dataclass
class Snapshot:
    """Flat graph state: row u holds deg[u] entries in ascending (dist, id) order."""
    ids: np.ndarray    # int32 [N, W], -1 padded
    dist: np.ndarray   # float64 [N, W] (exact ints for uint8 data, float32 values for float data)
    flags: np.ndarray  # uint8 [N, W], 1 = "new"
    deg: np.ndarray    # int32 [N]

    def copy(self) -> "Snapshot":
        return Snapshot(self.ids.copy(), self.dist.copy(), self.flags.copy(), self.deg.copy())

    @staticmethod
    def empty(n: int, W: int) -> "Snapshot":
        return Snapshot(np.full((n, W), -1, np.int32), np.zeros((n, W), np.float64),
                        np.zeros((n, W), np.uint8), np.zeros(n, np.int32))


def mix64(z: int) -> int:
    return int(_load().orc_mix64(ctypes.c_uint64(z & (2**64 - 1))))


def draw(seed: int, u: int, j: int) -> int:
    return int(_load().orc_draw(ctypes.c_uint64(seed), ctypes.c_uint64(u), ctypes.c_uint64(j)))


def delta(X: np.ndarray, a: int, b: int) -> float:
    _chk(X)
    L = _load()
    return float(L.orc_delta(_p(X), ctypes.c_int64(X.shape[0]), ctypes.c_int32(X.shape[1]),
                             ctypes.c_int(_dt(X)), ctypes.c_int64(a), ctypes.c_int64(b)))


def random_ids(n: int, u: int, S: int, seed: int) -> np.ndarray:
    out = np.zeros(S, np.int32)
    rc = _load().orc_random_ids(ctypes.c_int64(n), ctypes.c_int64(u), ctypes.c_int32(S),
                                ctypes.c_uint64(seed), _p(out))
    assert rc == 0
    return out


def random_graph(X: np.ndarray, S: int, seed: int, W: int) -> Snapshot:
    _chk(X)
    n, d = X.shape
    s = Snapshot.empty(n, W)
    rc = _load().orc_random_graph(_p(X), ctypes.c_int64(n), ctypes.c_int32(d), ctypes.c_int(_dt(X)),
                                  ctypes.c_int32(S), ctypes.c_uint64(seed), ctypes.c_int32(W),
                                  _p(s.ids), _p(s.dist), _p(s.flags), _p(s.deg))
    assert rc == 0, rc
    return s


def update_neighbors_sync(X: np.ndarray, snap: Snapshot, R: int, use_flag_skip: bool = True):
    """One synchronous UpdateNeighbors round; returns (new snapshot, evals, proposals)."""
    _chk(X)
    n, d = X.shape
    s = snap.copy()
    W = s.ids.shape[1]
    ev = ctypes.c_int64(0)
    npr = ctypes.c_int64(0)
    rc = _load().orc_update_neighbors_sync(
        _p(X), ctypes.c_int64(n), ctypes.c_int32(d), ctypes.c_int(_dt(X)), ctypes.c_int32(R),
        ctypes.c_int32(W), _p(s.ids), _p(s.dist), _p(s.flags), _p(s.deg),
        ctypes.c_int(1 if use_flag_skip else 0), ctypes.byref(ev), ctypes.byref(npr))
    assert rc == 0, rc
    return s, ev.value, npr.value


def add_reverse_edges(snap: Snapshot, R: int) -> Snapshot:
    s = snap.copy()
    n, W = s.ids.shape
    rc = _load().orc_add_reverse_edges(ctypes.c_int64(n), ctypes.c_int32(R), ctypes.c_int32(W),
                                       _p(s.ids), _p(s.dist), _p(s.flags), _p(s.deg))
    assert rc == 0, rc
    return s


@dataclass
class BuildResult:
    snap: Snapshot
    round_evals: np.ndarray
    round_props: np.ndarray
    init_evals: int


def build_sync(X: np.ndarray, S: int, R: int, T1: int, T2: int, seed: int,
               use_flag_skip: bool = True, W: int | None = None, progress: bool = False) -> BuildResult:
    """progress=True prints one stderr line per finished round (for runs of several minutes)."""
    _chk(X)
    _load().orc_set_progress(ctypes.c_int(1 if progress else 0))
    n, d = X.shape
    W = R if W is None else W
    s = Snapshot.empty(n, W)
    rev = np.zeros(T1 * T2, np.int64)
    rpr = np.zeros(T1 * T2, np.int64)
    ie = ctypes.c_int64(0)
    rc = _load().orc_build_sync(
        _p(X), ctypes.c_int64(n), ctypes.c_int32(d), ctypes.c_int(_dt(X)), ctypes.c_int32(S),
        ctypes.c_int32(R), ctypes.c_int32(T1), ctypes.c_int32(T2), ctypes.c_uint64(seed),
        ctypes.c_int(1 if use_flag_skip else 0), ctypes.c_int32(W), _p(s.ids), _p(s.dist),
        _p(s.flags), _p(s.deg), _p(rev), _p(rpr), ctypes.byref(ie))
    assert rc == 0, rc
    return BuildResult(s, rev, rpr, ie.value)


def update_neighbors_blocks(X: np.ndarray, snap: Snapshot, R: int, nblocks: int):
    """One block-sequential UpdateNeighbors pass (nblocks runs of consecutive ids in turn; 1 = the
    synchronous round, n = Alg. 4's vertex order); returns (new snapshot, evals, proposals)."""
    _chk(X)
    n, d = X.shape
    s = snap.copy()
    W = s.ids.shape[1]
    ev = ctypes.c_int64(0)
    npr = ctypes.c_int64(0)
    rc = _load().orc_update_neighbors_blocks(
        _p(X), ctypes.c_int64(n), ctypes.c_int32(d), ctypes.c_int(_dt(X)), ctypes.c_int32(R),
        ctypes.c_int32(W), ctypes.c_int64(nblocks), _p(s.ids), _p(s.dist), _p(s.flags), _p(s.deg),
        ctypes.byref(ev), ctypes.byref(npr))
    assert rc == 0, rc
    return s, ev.value, npr.value


def build_blocks(X: np.ndarray, S: int, R: int, T1: int, T2: int, seed: int, nblocks: int,
                 W: int | None = None, progress: bool = False) -> BuildResult:
    """Alg. 6 with block-sequential passes (see update_neighbors_blocks)."""
    _chk(X)
    _load().orc_set_progress(ctypes.c_int(1 if progress else 0))
    n, d = X.shape
    W = R if W is None else W
    s = Snapshot.empty(n, W)
    rev = np.zeros(T1 * T2, np.int64)
    rpr = np.zeros(T1 * T2, np.int64)
    rc = _load().orc_build_blocks(
        _p(X), ctypes.c_int64(n), ctypes.c_int32(d), ctypes.c_int(_dt(X)), ctypes.c_int32(S),
        ctypes.c_int32(R), ctypes.c_int32(T1), ctypes.c_int32(T2), ctypes.c_uint64(seed),
        ctypes.c_int64(nblocks), ctypes.c_int32(W), _p(s.ids), _p(s.dist), _p(s.flags), _p(s.deg),
        _p(rev), _p(rpr))
    assert rc == 0, rc
    return BuildResult(s, rev, rpr, n * S)


def build_wide(X: np.ndarray, S: int, R: int, M: int, T1: int, T2: int, seed: int) -> BuildResult:
    """Alg. 6 with synchronous rounds whose merges cut to M >= R entries; AddReverseEdges cuts to R.
    Rows of the result are M wide."""
    _chk(X)
    n, d = X.shape
    s = Snapshot.empty(n, M)
    rev = np.zeros(T1 * T2, np.int64)
    rpr = np.zeros(T1 * T2, np.int64)
    rc = _load().orc_build_wide(
        _p(X), ctypes.c_int64(n), ctypes.c_int32(d), ctypes.c_int(_dt(X)), ctypes.c_int32(S),
        ctypes.c_int32(R), ctypes.c_int32(M), ctypes.c_int32(T1), ctypes.c_int32(T2), ctypes.c_uint64(seed),
        ctypes.c_int32(M), _p(s.ids), _p(s.dist), _p(s.flags), _p(s.deg), _p(rev), _p(rpr))
    assert rc == 0, rc
    return BuildResult(s, rev, rpr, n * S)


def build_paper_order(X: np.ndarray, S: int, R: int, T1: int, T2: int, seed: int, W: int):
    """Alg. 6 in the paper's in-place vertex order; returns (ids, deg, evals, max_degree)."""
    _chk(X)
    n, d = X.shape
    ids = np.full((n, W), -1, np.int32)
    deg = np.zeros(n, np.int32)
    ev = ctypes.c_int64(0)
    mx = ctypes.c_int32(0)
    rc = _load().orc_build_paper_order(
        _p(X), ctypes.c_int64(n), ctypes.c_int32(d), ctypes.c_int(_dt(X)), ctypes.c_int32(S),
        ctypes.c_int32(R), ctypes.c_int32(T1), ctypes.c_int32(T2), ctypes.c_uint64(seed),
        ctypes.c_int32(W), _p(ids), _p(deg), ctypes.byref(ev), ctypes.byref(mx))
    assert rc == 0, rc
    return ids, deg, ev.value, mx.value


def rng_strategy(X: np.ndarray, u: int, cand: np.ndarray) -> np.ndarray:
    _chk(X)
    n, d = X.shape
    cand = np.ascontiguousarray(cand, np.int32)
    out = np.zeros(max(1, cand.size), np.int32)
    m = ctypes.c_int32(0)
    rc = _load().orc_rng_strategy(_p(X), ctypes.c_int64(n), ctypes.c_int32(d), ctypes.c_int(_dt(X)),
                                  ctypes.c_int64(u), _p(cand), ctypes.c_int32(cand.size), _p(out),
                                  ctypes.byref(m))
    assert rc == 0
    return out[:m.value].copy()


def bruteforce_knn(X: np.ndarray, Q: np.ndarray, k: int) -> np.ndarray:
    _chk(X), _chk(Q)
    assert Q.dtype == X.dtype and Q.shape[1] == X.shape[1]
    out = np.zeros((Q.shape[0], k), np.int32)
    rc = _load().orc_bruteforce_knn(_p(X), ctypes.c_int64(X.shape[0]), ctypes.c_int32(X.shape[1]),
                                    ctypes.c_int(_dt(X)), _p(Q), ctypes.c_int64(Q.shape[0]),
                                    ctypes.c_int32(k), _p(out))
    assert rc == 0
    return out


def search(X: np.ndarray, ids: np.ndarray, deg: np.ndarray, Q: np.ndarray, L: int, K: int, k: int,
           seed: int = 7):
    """Alg. 1 with the top-K out-degree cap; returns (ids [nq, k], distance evaluations)."""
    _chk(X), _chk(Q)
    ids = np.ascontiguousarray(ids, np.int32)
    deg = np.ascontiguousarray(deg, np.int32)
    out = np.zeros((Q.shape[0], k), np.int32)
    ev = ctypes.c_int64(0)
    rc = _load().orc_search(_p(X), ctypes.c_int64(X.shape[0]), ctypes.c_int32(X.shape[1]),
                            ctypes.c_int(_dt(X)), _p(ids), _p(deg), ctypes.c_int32(ids.shape[1]),
                            _p(Q), ctypes.c_int64(Q.shape[0]), ctypes.c_int32(L), ctypes.c_int32(K),
                            ctypes.c_int32(k), ctypes.c_uint64(seed), _p(out), ctypes.byref(ev))
    assert rc == 0
    return out, ev.value


def recall_at_k(found: np.ndarray, truth: np.ndarray) -> float:
    """|found row ∩ truth row| / k averaged over queries."""
    k = truth.shape[1]
    hit = 0
    for f, t in zip(found, truth):
        hit += len(set(f.tolist()) & set(t.tolist()))
    return hit / (k * truth.shape[0])
