"""rnnd_build_wide against the oracle's build_wide: UpdateNeighbors merges cut to M >= R entries, only
AddReverseEdges cuts to R (the paper bounds degrees nowhere else).  Exact comparison, M-wide rows."""
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


def cuda(a):
    import torch
    return torch.from_numpy(a).cuda()


def _data(kind, n, d, seed):
    if kind in ("gauss_u8", "unit_f32", "heavy_u8"):
        return wl.custom(kind, n, d, seed)
    g = np.random.default_rng(seed)
    if kind == "dense_u8":          # three tight clusters: lists grow to the cap
        c = g.integers(20, 236, size=(3, d))
        return np.clip(c[g.integers(0, 3, size=n)] + g.integers(-9, 10, size=(n, d)), 0, 255).astype(np.uint8)
    return (g.integers(-2, 3, size=(n, d)) * 0.25).astype(np.float32)


CASES = [
    # kind, N, d, S, R, M, T1, T2
    ("dense_u8", 900, 64, 8, 12, 128, 3, 3),
    ("dense_u8", 900, 64, 8, 12, 40, 3, 3),
    ("dense_u8", 900, 128, 16, 16, 17, 2, 4),
    ("heavy_u8", 3000, 128, 20, 24, 96, 3, 4),
    ("gauss_u8", 2000, 33, 6, 8, 64, 3, 3),
    ("unit_f32", 2500, 96, 10, 12, 96, 3, 3),
    ("unit_f32", 2500, 96, 10, 12, 128, 2, 3),
    ("lattice_f32", 800, 16, 10, 16, 100, 3, 2),
    ("gauss_u8", 1500, 64, 5, 5, 5, 2, 3),
]


@pytest.mark.parametrize("kind,N,d,S,R,M,T1,T2", CASES)
def test_build_wide_equals_oracle(rn, oracle_mod, kind, N, d, S, R, M, T1, T2):
    X = _data(kind, N, d, 40 + N + M)
    isf = X.dtype == np.float32
    want = oracle_mod.build_wide(X, S, R, M, T1, T2, 13)
    graph, degree, keys, st = rn.rnnd_build_wide(cuda(X), S, R, M, T1, T2, 13)
    assert_snapshot_equal(want.snap, isf, keys, degree, "%s N %d R %d M %d" % (kind, N, R, M))
    assert (graph.cpu().numpy() == want.snap.ids).all()
    assert list(st.algo_evals[:T1 * T2]) == want.round_evals.tolist()
    assert list(st.proposals[:T1 * T2]) == want.round_props.tolist()
    if M == R:
        g0, d0 = rn.rnnd_build(cuda(X), S, R, T1, T2, 13)
        assert (g0 == graph).all() and (d0 == degree).all()


def test_wide_rows_outgrow_R_and_reverse_edges_cut_them(rn):
    """Between AddReverseEdges calls a list may exceed R (up to M); right after a call it may not."""
    X = _data("dense_u8", 900, 64, 3)
    R, M = 12, 128
    _, deg_end, _, _ = rn.rnnd_build_wide(cuda(X), 8, R, M, 2, 3, 1)          # ends with UpdateNeighbors rounds
    assert int(deg_end.max()) > R
    g, deg1, keys, _ = rn.rnnd_build_wide(cuda(X), 8, R, M, 1, 3, 1)
    rn.rnnd_add_reverse_edges(keys[:, :M].contiguous(), deg1, M)                # plain call: cap = stride = M
    assert int(deg1.max()) <= M


def test_reverse_edges_cut_a_long_list_that_receives_nothing(rn, oracle_mod):
    """Alg. 5's first loop cuts EVERY out-list to its R shortest, also the list of a vertex no edge points to.
    Rows are M = 64 wide, R = 12; vertices 0 .. 5 hold 40 entries each and appear in nobody's list (their unions
    exceed 32 keys, so they take the one-vertex-at-a-time path of the union kernel), everyone else holds a short
    list among the ids >= 6.  Step-wise call on the snapshot, against the oracle's AddReverseEdges on M-wide rows."""
    from gpu_util import snapshot_to_device
    g = np.random.default_rng(5)
    n, d, R, M, lonely = 400, 32, 12, 64, 6
    X = np.clip(128 + g.normal(0, 30, size=(n, d)), 0, 255).astype(np.uint8)
    Xl = X.astype(np.int64)
    snap = oracle_mod.Snapshot.empty(n, M)
    for u in range(n):
        m = 40 if u < lonely else int(g.integers(0, 9))
        ids = g.choice(np.arange(lonely, n)[np.arange(lonely, n) != u], size=m, replace=False)
        dist = ((Xl[ids] - Xl[u]) ** 2).sum(1)
        order = np.lexsort((ids, dist))
        snap.ids[u, :m], snap.dist[u, :m] = ids[order], dist[order]
        snap.flags[u, :m] = g.integers(0, 2, size=m)
        snap.deg[u] = m
    want = oracle_mod.add_reverse_edges(snap, R)
    assert (want.deg[:lonely] == R).all() and want.deg.max() <= R       # the oracle cuts them (Alg. 5, first loop)
    keys, deg = snapshot_to_device(snap, False, M)
    rn.rnnd_add_reverse_edges_wide(keys, deg, R)
    assert_snapshot_equal(want, False, keys, deg, "lonely long lists")


def test_no_dropped_entry_means_the_unbounded_build(rn, oracle_mod):
    """The paper's UpdateNeighbors never drops an edge for lack of room (Sec. 4.4); rows here are at most 128
    slots wide.  The build counts the entries its merges had to drop (stats.dropped): where the count is zero in
    every round, the graph must be the one lists without any bound give -- the oracle with rows N - 1 wide.  And
    where lists are cut (rows only R wide on the same data), the count must say so."""
    X = _data("dense_u8", 900, 64, 3)
    n, S, R, T1, T2 = len(X), 8, 12, 3, 3
    unbounded = oracle_mod.build_wide(X, S, R, n - 1, T1, T2, 1)        # a list cannot hold more than N - 1 entries
    longest = int(unbounded.snap.deg.max())
    assert R < longest <= 128                                            # lists outgrow R, but fit 128 slots
    graph, degree, keys, st = rn.rnnd_build_wide(cuda(X), S, R, 128, T1, T2, 1)
    assert sum(st.dropped[:T1 * T2]) == 0
    import oracle
    cut = oracle.Snapshot(unbounded.snap.ids[:, :128].copy(), unbounded.snap.dist[:, :128].copy(),
                          unbounded.snap.flags[:, :128].copy(), unbounded.snap.deg.copy())
    assert_snapshot_equal(cut, False, keys, degree, "rows of 128 slots against unbounded lists")
    assert list(st.algo_evals[:T1 * T2]) == unbounded.round_evals.tolist()
    # rows only R wide: entries are dropped, and counted
    _, _, _, st_r = rn.rnnd_build_ex(cuda(X), S, R, T1, T2, 1)
    assert sum(st_r.dropped[:T1 * T2]) > 0
    # an intermediate width that still cuts somewhere during the build
    narrow = max(R + 1, longest // 2)
    want = oracle_mod.build_wide(X, S, R, narrow, T1, T2, 1)
    g2, d2, k2, st2 = rn.rnnd_build_wide(cuda(X), S, R, narrow, T1, T2, 1)
    assert_snapshot_equal(want.snap, False, k2, d2, "rows of %d slots" % narrow)
    print("longest unbounded list %d; dropped with rows of %d slots: %d, of %d slots: %d"
          % (longest, R, sum(st_r.dropped[:T1 * T2]), narrow, sum(st2.dropped[:T1 * T2])))
