"""Method-behaviour regression checks on the GPU path (Sec. 5.3, 5.4 and App. B of the paper): at a constant number of
UpdateNeighbors rounds T1*T2, a build without any AddReverseEdges call (T1 = 1) searches clearly worse
than the paper's T1 = 4, T2 = 15, and the in-degree bound of Alg. 5 holds on the final graph."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rn():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2310_20419_amd as m
    m.load_library()
    return m


def test_reverse_edges_matter_cfg2(rn, oracle_mod):
    import torch
    c = wl.CONFIGS["cfg2"]
    X = wl.make_data(c)
    Q = wl.make_queries(c, 200)
    Xd, Qd = torch.from_numpy(X).cuda(), torch.from_numpy(Q).cuda()
    truth = oracle_mod.bruteforce_knn(X, Q, 10)
    recall = {}
    for T1, T2 in ((1, 60), (4, 15)):
        graph, degree = rn.rnnd_build(Xd, c.S, c.R, T1, T2, wl.BUILD_SEED)
        ids, _, _ = rn.rnnd_search(Xd, graph, degree, Qd, 32, 32, 10, 7)
        recall[T1] = oracle_mod.recall_at_k(ids.cpu().numpy(), truth)
        g, dg = graph.cpu().numpy(), degree.cpu().numpy()
        assert dg.max() <= c.R
        if T1 == 1:
            assert dg.min() >= 1      # the nearest entry of a list is never pruned; only Alg. 5 can empty a list
        if T1 > 1:
            # the in-degree cut of Alg. 5 bounds the in-degree after each call; UpdateNeighbors never raises a vertex's
            # in-degree above what it was (a redirected edge replaces an edge into the same vertex)
            indeg = np.bincount(g[g >= 0], minlength=c.N)
            assert indeg.max() <= c.R
    print("recall@10 at L=32, K=32: T1=1 %.4f, T1=4 %.4f" % (recall[1], recall[4]))
    assert recall[4] > 0.93
    assert recall[4] > recall[1] + 0.03


SWEEP = [(1, 60), (2, 30), (4, 15), (12, 5), (60, 1)]


def test_t1_t2_sweep_at_constant_rounds_cfg2(rn, oracle_mod):
    """Sec. 5.4: (T1, T2) varied at T1 * T2 = 60 on cfg2, GPU build + GPU search (500 queries, L = 32, K = 32).
    What the paper reports and this data reproduces: without AddReverseEdges (T1 = 1) the graph searches clearly
    worse than any setting with T1 >= 2 and T2 > 1, and among those the choice matters little.  What this data
    adds: the other extreme, T2 = 1 (an AddReverseEdges call after every single round), is worse still -- so
    'T1 = 1 is the worst setting' holds among the settings with T2 > 1, which are the ones the paper sweeps."""
    import torch
    c = wl.CONFIGS["cfg2"]
    X = wl.make_data(c)
    Q = wl.make_queries(c, 500)
    Xd, Qd = torch.from_numpy(X).cuda(), torch.from_numpy(Q).cuda()
    truth = oracle_mod.bruteforce_knn(X, Q, 10)
    recall, evals, mean_deg = {}, {}, {}
    for T1, T2 in SWEEP:
        graph, degree = rn.rnnd_build(Xd, c.S, c.R, T1, T2, wl.BUILD_SEED)
        ids, _, ev = rn.rnnd_search(Xd, graph, degree, Qd, 32, 32, 10, 7)
        recall[T1] = oracle_mod.recall_at_k(ids.cpu().numpy(), truth)
        evals[T1] = ev / len(Q)
        mean_deg[T1] = float(degree.float().mean())
        g, dg = graph.cpu().numpy(), degree.cpu().numpy()
        assert dg.max() <= c.R
        if T1 > 1:
            assert np.bincount(g[g >= 0], minlength=c.N).max() <= c.R        # Sec. 5.3: in-degree at most R
    print("recall@10 / evaluations per query / mean out-degree by (T1, T2): "
          + ", ".join("(%d,%d) %.3f / %.0f / %.2f" % (a, b, recall[a], evals[a], mean_deg[a]) for a, b in SWEEP))
    middle = [recall[2], recall[4], recall[12]]
    assert min(middle) > recall[1] + 0.05                     # T1 = 1 is clearly worse than every 2 <= T1 <= 12
    assert max(middle) - min(middle) < 0.02                   # ... among which the choice matters little
    assert recall[60] < recall[1]                             # T2 = 1 is worse still on this data (see docstring)
    assert min(middle) > 0.95


def test_degree_distribution_cfg2(rn):
    """Sec. 5.3 and App. B on cfg2: the average out-degree is far below R, every in-degree is at most R, and with
    the paper's unbounded UpdateNeighbors merges (rows wider than R, rnnd_build_wide) some out-degrees end up
    above R (the paper reports maxima around 150 for R = 96 on its datasets).  The average out-degree under the
    search cap K of Eq. 4 -- the paper's AOD table -- is mean(min(degree, K)): it grows with K and reaches the
    plain average once K covers the longest list."""
    import torch
    c = wl.CONFIGS["cfg2"]
    Xd = torch.from_numpy(wl.make_data(c)).cuda()
    graph, degree = rn.rnnd_build(Xd, c.S, c.R, c.T1, c.T2, wl.BUILD_SEED)
    g, dg = graph.cpu().numpy(), degree.cpu().numpy()
    indeg = np.bincount(g[g >= 0], minlength=c.N)
    aod = {K: float(np.minimum(dg, K).mean()) for K in (16, 32, 48, 64, 96)}
    print("cfg2: mean out-degree %.2f, max %d; max in-degree %d; AOD by K %s" % (dg.mean(), dg.max(), indeg.max(), aod))
    assert 6.0 < dg.mean() < 30.0 and dg.mean() < c.R / 3           # "far below R" (paper: about 20 of 96)
    assert dg.max() <= c.R and indeg.max() <= c.R          # (a list can end up empty: every target may cut the edge, Alg. 5)
    assert indeg.sum() == dg.sum()
    ks = sorted(aod)
    assert all(aod[a] <= aod[b] for a, b in zip(ks, ks[1:])) and abs(aod[96] - dg.mean()) < 1e-9
    assert aod[16] < dg.mean()                                        # the cap bites: some lists are longer than 16
    # the paper's arrangement: only AddReverseEdges bounds the degrees
    gw, dw, _, _ = rn.rnnd_build_wide(Xd, c.S, c.R, 128, c.T1, c.T2, wl.BUILD_SEED, want_keys=False)
    dwn = dw.cpu().numpy()
    gwn = gw.cpu().numpy()
    print("cfg2, rows 128 wide: mean out-degree %.2f, max %d, lists longer than R: %d"
          % (dwn.mean(), dwn.max(), int((dwn > c.R).sum())))
    assert dwn.max() > c.R and dwn.mean() >= dg.mean()
    # in-degrees: bounded by R right after the last AddReverseEdges and never raised by UpdateNeighbors
    assert np.bincount(gwn[gwn >= 0], minlength=c.N).max() <= c.R
