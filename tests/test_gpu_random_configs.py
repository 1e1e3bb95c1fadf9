"""Seeded random small configurations (shapes, dtypes and parameters that no named workload has):
full build and search, GPU against the oracle, everything identical."""
import numpy as np
import pytest

import workloads as wl
from gpu_util import assert_snapshot_equal

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rn():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2310_20419_amd as m
    m.load_library()
    return m


def _data(kind, n, d, seed):
    """The named generators where they take any d; plus two tie-heavy ones made here."""
    if kind in ("gauss_u8", "unit_f32"):
        return wl.custom(kind, n, d, seed)
    g = np.random.default_rng(seed)
    if kind == "ties_u8":                       # few distinct values: many equal distances, duplicates
        return g.integers(0, 3, size=(n, d)).astype(np.uint8) * 100
    return (g.integers(-2, 3, size=(n, d)) * 0.25).astype(np.float32)    # lattice_f32: exact ties in float


def _configs():
    g = np.random.default_rng(20419)
    out = []
    dims = [1, 2, 3, 7, 16, 17, 32, 48, 64, 96, 100, 128, 160, 256]
    for i in range(96):
        N = int(g.choice([2, 3, 5, 9, 33, 65, 130, 257, 400, 900, 1500, 3000]))
        d = int(g.choice(dims))
        kind = str(g.choice(["gauss_u8", "ties_u8", "unit_f32", "lattice_f32"]))
        R = int(g.choice([1, 2, 5, 8, 9, 16, 17, 31, 32, 33, 48, 64, 65, 96, 97, 128]))
        S = int(g.integers(1, min(R, N - 1) + 1))
        T1, T2 = int(g.integers(1, 4)), int(g.integers(1, 5))
        out.append((i, kind, N, d, S, R, T1, T2))
    return out


@pytest.mark.parametrize("i,kind,N,d,S,R,T1,T2", _configs())
def test_random_config(rn, oracle_mod, i, kind, N, d, S, R, T1, T2):
    import torch
    X = _data(kind, N, d, 1000 + i)
    isf = X.dtype == np.float32
    want = oracle_mod.build_sync(X, S, R, T1, T2, 5 + i)
    Xd = torch.from_numpy(X).cuda()
    graph, degree, keys, st = rn.rnnd_build_ex(Xd, S, R, T1, T2, 5 + i)
    assert_snapshot_equal(want.snap, isf, keys, degree, "config %d" % i)
    assert (graph.cpu().numpy() == want.snap.ids).all()
    assert list(st.algo_evals[:T1 * T2]) == want.round_evals.tolist()
    # search on it
    Q = _data(kind, 11, d, 2000 + i)
    L = int(min(128, max(1, [3, 16, 64, 128][i % 4])))
    K = [1, 4, 32, 200][(i // 4) % 4]
    k = min(L, 10)
    found, _, evals = rn.rnnd_search(Xd, graph, degree, torch.from_numpy(Q).cuda(), L, K, k, 99 + i)
    wfound, wevals = oracle_mod.search(X, want.snap.ids, want.snap.deg, Q, L, K, k, 99 + i)
    assert (found.cpu().numpy() == wfound).all() and evals == wevals


def _mid_configs():
    g = np.random.default_rng(31415)
    out = []
    for i in range(16):
        N = int(g.choice([5000, 12000, 20000]))
        kind, d = [("heavy_u8", 128), ("heavy_u8", 64), ("gauss_u8", 32), ("gauss_u8", 48), ("unit_f32", 96),
                   ("unit_f32", 32), ("ties_u8", 16), ("lattice_f32", 16)][i % 8]
        R = int(g.choice([8, 16, 32, 64, 96]))
        S = int(g.integers(max(1, R // 4), R + 1))
        out.append((i, kind, N, d, S, R, int(g.integers(2, 4)), int(g.integers(2, 6))))
    return out


@pytest.mark.parametrize("i,kind,N,d,S,R,T1,T2", _mid_configs())
def test_mid_size_config(rn, oracle_mod, i, kind, N, d, S, R, T1, T2):
    """Tens of thousands of vertices with small degree caps: hubs overflow the inboxes, Alg. 5's in-degree cap
    bites, lists fill up to R."""
    import torch
    X = _data(kind, N, d, 3000 + i) if kind != "heavy_u8" else wl.custom(kind, N, d, 3000 + i)
    isf = X.dtype == np.float32
    want = oracle_mod.build_sync(X, S, R, T1, T2, 50 + i)
    graph, degree, keys, st = rn.rnnd_build_ex(torch.from_numpy(X).cuda(), S, R, T1, T2, 50 + i)
    assert_snapshot_equal(want.snap, isf, keys, degree, "mid config %d" % i)
    assert list(st.algo_evals[:T1 * T2]) == want.round_evals.tolist()
    assert list(st.proposals[:T1 * T2]) == want.round_props.tolist()
