"""AddReverseEdges' two ways of transposing the edge set (one arrival-number atomic per edge; binned by target
range without device-scope atomics per edge) must both give the oracle's result.  The default picks by size, so
the small parity tests exercise the first and the 1M / 20M tests the second; here each is forced on the same
inputs: ordinary graphs, a hub that receives hundreds of reversed edges (inbox overflow into bins), rows wider
than R, several ranges of targets, and empty lists."""
import numpy as np
import pytest

import workloads as wl
from gpu_util import assert_snapshot_equal, snapshot_to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rn():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2310_20419_amd as m
    m.load_library()
    return m


@pytest.fixture(params=[1, 2], ids=["atomics", "binned"])
def path(request, rn):
    rn.rnnd_set_transpose_path(request.param)
    yield request.param
    rn.rnnd_set_transpose_path(0)


def cuda(a):
    import torch
    return torch.from_numpy(a).cuda()


@pytest.mark.parametrize("kind,n,d,S,R", [("heavy_u8", 3000, 128, 20, 96), ("gauss_u8", 9000, 32, 10, 16),
                                          ("unit_f32", 2500, 96, 12, 24), ("heavy_u8", 20000, 128, 6, 8)])
def test_step_by_step_from_oracle_snapshots(rn, oracle_mod, path, kind, n, d, S, R):
    X = wl.custom(kind, n, d, 21)
    isf = X.dtype == np.float32
    Xd = cuda(X)
    snap = oracle_mod.random_graph(X, S, 77, R)
    for step in ["r", "u", "u", "r", "u", "r", "r"]:
        keys, deg = snapshot_to_device(snap, isf, R)
        if step == "u":
            snap, _, _ = oracle_mod.update_neighbors_sync(X, snap, R)
            rn.rnnd_update_neighbors(Xd, keys, deg, R, 1)
        else:
            snap = oracle_mod.add_reverse_edges(snap, R)
            rn.rnnd_add_reverse_edges(keys, deg, R)
        assert_snapshot_equal(snap, isf, keys, deg, "%s step %s" % (kind, step), float_bar=False)


def test_hub_and_empty_lists(rn, oracle_mod, path):
    """Vertex 0 is in almost every list and vertex 1 in several hundred (reversed edges beyond an inbox: the bins), vertices
    5000 .. 5999 hold nothing and are in nobody's list, and the ids span five ranges of 2,048 targets."""
    g = np.random.default_rng(3)
    n, R = 9000, 16
    X = np.clip(128 + g.normal(0, 40, size=(n, 32)), 0, 255).astype(np.uint8)
    Xl = X.astype(np.int64)
    snap = oracle_mod.Snapshot.empty(n, R)
    live = np.concatenate([np.arange(1, 5000), np.arange(6000, n)])
    for u in range(n):
        if 5000 <= u < 6000:
            continue
        m = int(g.integers(1, 9))
        ids = g.choice(live[live != u], size=m, replace=False)
        if u != 0 and g.random() < 0.9:
            ids[0] = 0                      # thousands of edges into vertex 0: beyond the binned path's LDS stash
        if u > 1 and m > 1 and g.random() < 0.07:
            ids[1] = 1                      # several hundred into vertex 1: inside it
        ids = np.unique(ids)
        dist = ((Xl[ids] - Xl[u]) ** 2).sum(1)
        order = np.lexsort((ids, dist))
        m = len(ids)
        snap.ids[u, :m], snap.dist[u, :m], snap.deg[u] = ids[order], dist[order], m
        snap.flags[u, :m] = g.integers(0, 2, size=m)
    want = oracle_mod.add_reverse_edges(snap, R)
    keys, deg = snapshot_to_device(snap, False, R)
    rn.rnnd_add_reverse_edges(keys, deg, R)
    assert_snapshot_equal(want, False, keys, deg, "hub and empty lists")
    assert want.deg[0] == R and (want.deg[5000:6000] == 0).all()


def test_wide_rows(rn, oracle_mod, path):
    X = wl.custom("heavy_u8", 6000, 128, 5)
    want = oracle_mod.build_wide(X, 10, 12, 48, 3, 3, 13)
    graph, degree, keys, st = rn.rnnd_build_wide(cuda(X), 10, 12, 48, 3, 3, 13)
    assert_snapshot_equal(want.snap, False, keys, degree, "wide rows")


def test_full_builds(rn, oracle_mod, path):
    for name, n in (("cfg1", 5000), ("cfg2", 12000)):
        c = wl.CONFIGS[name]
        X = wl.make_data(c, n)
        want = oracle_mod.build_sync(X, c.S, c.R, c.T1, c.T2, wl.BUILD_SEED)
        graph, degree, keys, st = rn.rnnd_build_ex(cuda(X), c.S, c.R, c.T1, c.T2, wl.BUILD_SEED)
        assert_snapshot_equal(want.snap, False, keys, degree, name)
        wb = oracle_mod.build_blocks(X, c.S, c.R, 2, 3, wl.BUILD_SEED, 3)
        graph, degree, keys, st = rn.rnnd_build_blocks(cuda(X), c.S, c.R, 2, 3, wl.BUILD_SEED, 3)
        assert_snapshot_equal(wb.snap, False, keys, degree, name + " block-sequential")


def test_both_paths_agree_at_a_size_between_the_small_tests_and_the_full_ones(rn):
    """300,000 rows (above the size where the default switches to the binned path): the two forced paths and the
    default give one graph."""
    import torch
    c = wl.CONFIGS["cfg3"]
    Xd = cuda(wl.make_data(c, 300_000))
    out = []
    for p in (1, 2, 0):
        rn.rnnd_set_transpose_path(p)
        out.append(rn.rnnd_build(Xd, c.S, c.R, 3, 4, wl.BUILD_SEED))
    rn.rnnd_set_transpose_path(0)
    for g, d in out[1:]:
        assert (g == out[0][0]).all() and (d == out[0][1]).all()
