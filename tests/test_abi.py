"""CPU-side checks of the boundary: the library loads, exports every symbol include/rnnd.h declares,
and rejects bad arguments with the documented status codes before touching the GPU."""
import ctypes
import os

import pytest

import paper_2310_20419_amd as rn


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(rn.lib_path()):
        from paper_2310_20419_amd import build
        build.build()
    return rn.load_library()


def test_every_declared_symbol_is_exported(lib):
    names = rn.exported_symbols()
    assert {"rnnd_build", "rnnd_build_ex", "rnnd_random_graph", "rnnd_update_neighbors",
            "rnnd_add_reverse_edges", "rnnd_export_graph", "rnnd_search", "rnnd_workspace_bytes",
            "rnnd_strerror", "rnnd_version", "rnnd_set_kernel_variant", "rnnd_build_blocks",
            "rnnd_update_neighbors_blocks", "rnnd_probe_gather", "rnnd_build_wide", "rnnd_release_workspace",
            "rnnd_set_workspace_poison", "rnnd_set_event_timing", "rnnd_probe_gather_map", "rnnd_set_scan_launches"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_version_and_messages(lib):
    assert rn.rnnd_version() >= 100
    assert rn.rnnd_strerror(0) == "ok"
    for s in range(-7, 0):
        assert rn.rnnd_strerror(s) not in ("ok", "unknown status")
    assert rn.rnnd_strerror(-99) == "unknown status"


def test_bad_arguments_are_rejected_without_a_gpu(lib):
    one = ctypes.c_void_p(1)   # never dereferenced: validation comes first
    ok = dict(X=one, N=100, d=16, dtype=0, metric=0, S=4, R=8, T1=1, T2=1)

    def call(**kw):
        a = dict(ok, **kw)
        return lib.rnnd_build(a["X"], a["N"], a["d"], a["dtype"], a["metric"], a["S"], a["R"], a["T1"],
                              a["T2"], 0, a.get("g", one), a.get("deg", one), None)

    assert call(X=None) == -1 and call(g=None) == -1 and call(deg=None) == -1
    assert call(N=1) == -2 and call(d=0) == -2 and call(d=33026) == -2 and call(N=2**31 - 1) == -2
    assert call(S=0) == -3 and call(S=9) == -3 and call(R=0) == -3 and call(R=129) == -3
    assert call(T1=0) == -3 and call(T2=0) == -3 and call(N=5, S=5, R=8) == -3
    assert call(dtype=4) == -4 and call(dtype=-1) == -4 and call(metric=1) == -4
    assert call(N=50_000_000, R=128, S=4) == -2          # N*R does not fit the 32-bit slot counters
    assert call(N=25_000_000, R=96, S=4) == -2           # ... nor the signed bin offsets (N*R > 2^31 - 256)
    assert call(T1=400, T2=400) == -3                    # more rounds than counter blocks
    assert lib.rnnd_add_reverse_edges(25_000_000, 96, one, one, None) == -2
    assert lib.rnnd_add_reverse_edges(100, 8, None, one, None) == -1
    assert lib.rnnd_set_kernel_variant(7) == -3 and lib.rnnd_set_kernel_variant(3) == -3
    assert lib.rnnd_set_kernel_variant(0) == 0
    assert lib.rnnd_set_scan_launches(4) == -3 and lib.rnnd_set_scan_launches(-1) == -3 and lib.rnnd_set_scan_launches(0) == 0
    # block-sequential entry points: same checks, plus the number of runs
    def blocks(**kw):
        a = dict(ok, **kw)
        return lib.rnnd_build_blocks(a["X"], a["N"], a["d"], a["dtype"], a["metric"], a["S"], a["R"], a["T1"],
                                     a["T2"], 0, a.get("blocks", 4), a.get("g", one), a.get("deg", one), None, None,
                                     None)
    assert blocks(blocks=0) == -3 and blocks(blocks=101) == -3 and blocks(X=None) == -1 and blocks(g=None) == -1
    assert blocks(T1=400, T2=400, blocks=100) == -3 and blocks(S=0) == -3 and blocks(dtype=4) == -4
    assert lib.rnnd_update_neighbors_blocks(one, 100, 16, 0, 0, 8, one, one, 1, 0, None, None) == -3
    assert lib.rnnd_update_neighbors_blocks(one, 100, 16, 0, 0, 8, None, one, 1, 4, None, None) == -1
    assert lib.rnnd_update_neighbors_blocks(one, 100, 16, 0, 0, 8, one, one, 0, 4, None, None) == -3
    # wide merges: R <= M <= RNND_MAX_R
    def wide(R, M, X=one):
        return lib.rnnd_build_wide(X, 100, 16, 0, 0, 4, R, M, 1, 1, 0, one, one, None, None, None)
    assert wide(8, 7) == -3 and wide(8, 129) == -3 and wide(8, 0) == -3 and wide(8, 16, X=None) == -1
    # the gather probe
    import ctypes as c
    out = c.c_double(0)
    assert lib.rnnd_probe_gather(None, 10, 128, 100, 1, c.byref(out), None) == -1
    assert lib.rnnd_probe_gather(one, 10, 128, 100, 1, None, None) == -1
    assert lib.rnnd_probe_gather(c.c_void_p(16), 0, 128, 100, 1, c.byref(out), None) == -2
    assert lib.rnnd_probe_gather(c.c_void_p(16), 10, 100, 100, 1, c.byref(out), None) == -3      # not a multiple of 16
    assert lib.rnnd_probe_gather(c.c_void_p(8), 10, 128, 100, 1, c.byref(out), None) == -3       # misaligned
    lib.rnnd_probe_gather_map.argtypes = [c.c_void_p, c.c_int64, c.c_int64, c.c_int64, c.c_int, c.c_uint64,
                                          c.POINTER(c.c_double), c.c_void_p]
    assert lib.rnnd_probe_gather_map(None, 10, 128, 100, 2, 1, c.byref(out), None) == -1
    assert lib.rnnd_probe_gather_map(c.c_void_p(16), 10, 128, 100, 3, 1, c.byref(out), None) == -3   # 1, 2, 4 or 8 lanes
    assert lib.rnnd_probe_gather_map(c.c_void_p(16), 10, 128, 100, 0, 1, c.byref(out), None) == -3
    assert lib.rnnd_probe_gather_map(c.c_void_p(16), 10, 96, 100, 4, 1, c.byref(out), None) == -3    # 6 pieces, 4 lanes
    assert lib.rnnd_probe_gather_map(c.c_void_p(16), 10, 96, 100, 2, 1, c.byref(out), None) == -3    # 3 pieces per lane
    # rnnd_search: parameters are checked before pointers, pointers before any GPU call
    def search(**kw):
        a = dict(dict(X=one, N=100, d=16, dtype=0, metric=0, g=one, dg=one, W=8, Q=one, nq=3, L=16, K=8, k=5,
                      out=one), **kw)
        return lib.rnnd_search(a["X"], a["N"], a["d"], a["dtype"], a["metric"], a["g"], a["dg"], a["W"], a["Q"],
                               a["nq"], a["L"], a["K"], a["k"], 1, a["out"], None, None, None)
    assert search(L=0) == -3 and search(L=129) == -3 and search(K=0) == -3 and search(k=0) == -3
    assert search(k=17) == -3 and search(W=0) == -3 and search(nq=-1) == -2
    assert search(X=None) == -1 and search(g=None) == -1 and search(dg=None) == -1 and search(Q=None) == -1
    assert search(out=None) == -1 and search(dtype=4) == -4


def test_an_impossible_workspace_is_an_allocation_failure_without_a_gpu(lib):
    """N * R is inside the slot bound, but the workspace (about 1.4 TB) is beyond any device: RNND_ERR_OOM,
    decided before the first HIP call, so it is the same on a box without a GPU."""
    one = ctypes.c_void_p(1)
    n = 2**31 - 512
    assert rn.rnnd_workspace_bytes(n, 16, rn.RNND_U8, 1, 1) > 2**40
    assert lib.rnnd_build(one, n, 16, 0, 0, 1, 1, 1, 1, 0, one, one, None) == -5
    assert lib.rnnd_update_neighbors(one, n, 16, 0, 0, 1, one, one, 1, None, None) == -5
    assert lib.rnnd_add_reverse_edges(n, 1, one, one, None) == -5
    assert "memory" in rn.rnnd_strerror(-5)


def test_workspace_bytes(lib):
    b = rn.rnnd_workspace_bytes(1_000_000, 128, rn.RNND_U8, 96, 60)
    # the size grows with the number of rounds (one counter block each), and the query covers every
    # number of rounds a build accepts
    assert rn.rnnd_workspace_bytes(1_000_000, 128, rn.RNND_U8, 96, 131072) > b + 131000 * 2000
    with pytest.raises(rn.RnndError):
        rn.rnnd_workspace_bytes(1_000_000, 128, rn.RNND_U8, 96, 131073)
    # graph (8 B) + redirected-edge slots (16 B) + bins (8 B) per list slot, a 64-key inbox per vertex, and
    # (uint8 rows of 32/64/128 bytes) the int8 copy of X dominate; small per-vertex arrays on top
    per_vertex = 96 * 32 + 512 + 128
    assert 1_000_000 * per_vertex <= b < 1_000_000 * (per_vertex + 128)
    # float rows have no int8 copy
    bf = rn.rnnd_workspace_bytes(1_000_000, 96, rn.RNND_F32, 96, 60)
    assert 1_000_000 * (96 * 32 + 512) <= bf < 1_000_000 * (96 * 32 + 512 + 128)
    with pytest.raises(rn.RnndError):
        rn.rnnd_workspace_bytes(1_000_000, 128, rn.RNND_U8, 500, 60)


def test_key_packing_roundtrip():
    import numpy as np
    ids = np.array([[5, 9, -1], [2, -1, -1]], np.int32)
    bits = np.array([[10, 20, 0], [7, 0, 0]], np.uint32)
    flags = np.array([[1, 0, 0], [0, 0, 0]], np.uint8)
    deg = np.array([2, 1], np.int32)
    k = rn.pack_keys(ids, bits, flags, deg)
    assert k[0, 0] == (10 << 32) | (5 << 1) | 1 and k[0, 2] == 2**64 - 1
    i2, b2, f2 = rn.unpack_keys(k, deg)
    assert (i2 == ids).all() and (b2 == bits).all() and (f2 == flags).all()
