"""Block-sequential passes on the GPU (rnnd_build_blocks, rnnd_update_neighbors_blocks) against the
oracle's block-sequential variant: runs of consecutive vertex ids take their turn in id order and a run's
redirected edges are merged before the next run starts (Alg. 4 visits the vertices one after the
other and its edge update changes the edge set at once).  Every number of runs defines one graph per seed, so the
comparison is exact: ids, distances, flags, degrees and per-pass evaluation counts."""
import numpy as np
import pytest

import workloads as wl
from conftest import live
from gpu_util import assert_snapshot_equal, snapshot_to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rn():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2310_20419_amd as m
    m.load_library()
    return m


def cuda(a):
    import torch
    return torch.from_numpy(a).cuda()


def _data(kind, n, d, seed):
    if kind in ("gauss_u8", "unit_f32"):
        return wl.custom(kind, n, d, seed)
    g = np.random.default_rng(seed)
    if kind == "ties_u8":
        return g.integers(0, 3, size=(n, d)).astype(np.uint8) * 100
    return (g.integers(-2, 3, size=(n, d)) * 0.25).astype(np.float32)


CASES = [
    # kind, N, d, S, R, T1, T2, blocks
    ("gauss_u8", 2000, 128, 8, 24, 2, 3, 1),
    ("gauss_u8", 2000, 128, 8, 24, 2, 3, 2),
    ("gauss_u8", 2000, 128, 8, 24, 2, 3, 7),
    ("gauss_u8", 1500, 64, 10, 32, 2, 2, 1500),
    ("gauss_u8", 3001, 32, 12, 96, 3, 2, 16),
    ("gauss_u8", 900, 17, 5, 9, 2, 4, 13),
    ("ties_u8", 700, 3, 6, 16, 2, 3, 5),
    ("ties_u8", 300, 2, 4, 128, 2, 3, 300),
    ("unit_f32", 2000, 96, 8, 24, 2, 3, 3),
    ("unit_f32", 1200, 96, 20, 96, 2, 3, 1200),
    ("unit_f32", 2500, 160, 12, 48, 2, 2, 10),
    ("unit_f32", 800, 7, 6, 33, 2, 3, 9),
    ("lattice_f32", 600, 3, 6, 16, 2, 3, 4),
    ("lattice_f32", 257, 16, 9, 128, 3, 2, 257),
    ("gauss_u8", 2, 128, 1, 1, 1, 2, 2),
    ("gauss_u8", 5, 32, 4, 4, 2, 2, 3),
]


@pytest.mark.parametrize("kind,N,d,S,R,T1,T2,blocks", CASES)
def test_build_blocks_equals_oracle(rn, oracle_mod, kind, N, d, S, R, T1, T2, blocks):
    X = _data(kind, N, d, 77 + N + blocks)
    isf = X.dtype == np.float32
    want = oracle_mod.build_blocks(X, S, R, T1, T2, 11, blocks)
    graph, degree, keys, st = rn.rnnd_build_blocks(cuda(X), S, R, T1, T2, 11, blocks)
    assert_snapshot_equal(want.snap, isf, keys, degree, "%s N %d blocks %d" % (kind, N, blocks))
    assert (graph.cpu().numpy() == want.snap.ids).all()
    assert list(st.algo_evals[:T1 * T2]) == want.round_evals.tolist()
    assert list(st.proposals[:T1 * T2]) == want.round_props.tolist()


def test_one_block_is_the_synchronous_build(rn):
    c = wl.CONFIGS["cfg1"]
    X = wl.make_data(c)
    g0, d0 = rn.rnnd_build(cuda(X), c.S, c.R, c.T1, c.T2, wl.BUILD_SEED)
    g1, d1, _, _ = rn.rnnd_build_blocks(cuda(X), c.S, c.R, c.T1, c.T2, wl.BUILD_SEED, 1)
    assert (g0 == g1).all() and (d0 == d1).all()
    g4, d4, _, _ = rn.rnnd_build_blocks(cuda(X), c.S, c.R, c.T1, c.T2, wl.BUILD_SEED, 4)
    assert (g4 != g1).any()          # the order of the vertex loop matters


@pytest.mark.parametrize("blocks", [3, 64, 5000])
def test_cfg1_build_blocks(rn, oracle_mod, blocks):
    c = wl.CONFIGS["cfg1"]
    X = wl.make_data(c)
    want = oracle_mod.build_blocks(X, c.S, c.R, c.T1, c.T2, wl.BUILD_SEED, blocks)
    graph, degree, keys, st = rn.rnnd_build_blocks(cuda(X), c.S, c.R, c.T1, c.T2, wl.BUILD_SEED, blocks)
    assert_snapshot_equal(want.snap, False, keys, degree, "cfg1 blocks %d" % blocks)
    assert list(st.algo_evals[:c.T1 * c.T2]) == want.round_evals.tolist()


def test_stepwise_passes_from_an_oracle_snapshot(rn, oracle_mod):
    """One pass at a time from a snapshot the oracle made (after RandomGraph, rounds and a reverse call)."""
    X = _data("gauss_u8", 1800, 128, 5)
    R = 40
    snap = oracle_mod.random_graph(X, 10, 3, R)
    snap, _, _ = oracle_mod.update_neighbors_sync(X, snap, R)
    snap = oracle_mod.add_reverse_edges(snap, R)
    for blocks in (1, 6, 1800):
        keys, deg = snapshot_to_device(snap, False, R)
        want = snap
        for p in range(3):
            want, evals, props = oracle_mod.update_neighbors_blocks(X, want, R, blocks)
            st = rn.rnnd_update_neighbors_blocks(cuda(X), keys, deg, R, blocks, 1)
            assert_snapshot_equal(want, False, keys, deg, "blocks %d pass %d" % (blocks, p))
            assert st.algo_evals[0] == evals and st.proposals[0] == props


@live
def test_cfg2_build_blocks_and_search_quality(rn, oracle_mod):
    """Workload cfg2 (100,000 x 128 uint8) in 16 runs per pass: identical to the oracle's 16-run build, and
    the graph searches as well as the synchronous one (statistical: recall@10 within 0.01)."""
    c = wl.CONFIGS["cfg2"]
    X = wl.make_data(c)
    Xd = cuda(X)
    want = oracle_mod.build_blocks(X, c.S, c.R, c.T1, c.T2, wl.BUILD_SEED, 16, progress=True)
    graph, degree, keys, st = rn.rnnd_build_blocks(Xd, c.S, c.R, c.T1, c.T2, wl.BUILD_SEED, 16)
    assert_snapshot_equal(want.snap, False, keys, degree, "cfg2 blocks 16")
    assert list(st.algo_evals[:60]) == want.round_evals.tolist()
    Q = wl.make_queries(c, 500)
    truth = oracle_mod.bruteforce_knn(X, Q, 10)
    g0, d0 = rn.rnnd_build(Xd, c.S, c.R, c.T1, c.T2, wl.BUILD_SEED)
    rec = {}
    for name, (g, dg) in {"sync": (g0, d0), "blocks16": (graph, degree)}.items():
        ids, _, _ = rn.rnnd_search(Xd, g, dg, cuda(Q), 64, 32, 10, 7)
        rec[name] = oracle_mod.recall_at_k(ids.cpu().numpy(), truth)
    print("recall@10 L=64 K=32: synchronous %.4f, 16 runs per pass %.4f" % (rec["sync"], rec["blocks16"]))
    assert abs(rec["sync"] - rec["blocks16"]) < 0.01


def test_bad_block_counts_are_rejected(rn):
    X = cuda(_data("gauss_u8", 100, 32, 1))
    for blocks in (0, -1, 101):
        with pytest.raises(rn.RnndError):
            rn.rnnd_build_blocks(X, 4, 8, 1, 1, 0, blocks)
    with pytest.raises(rn.RnndError):                 # more run slots than the library keeps counters for
        rn.rnnd_build_blocks(X, 4, 8, 100, 100, 0, 100)
