"""GPU search (Alg. 1 with the out-degree cap of Eq. 4) against the CPU oracle's search on the same
graph, queries, L, K, k and seed, through the C ABI: result ids, their distances and the number of
distance evaluations must be identical (uint8 and float32: both sides accumulate float distances in
double and round once)."""
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


def cuda(a):
    import torch
    return torch.from_numpy(a).cuda()


def built(rn, X, S, R, T1, T2):
    graph, degree = rn.rnnd_build(cuda(X), S, R, T1, T2, wl.BUILD_SEED)
    return graph, degree


def check(rn, oracle_mod, X, graph, degree, Q, L, K, k, seed, label):
    ids, dist, ev = rn.rnnd_search(cuda(X), graph, degree, cuda(Q), L, K, k, seed, want_dist=True)
    want, wev = oracle_mod.search(X, graph.cpu().numpy(), degree.cpu().numpy(), Q, L, K, k, seed)
    got = ids.cpu().numpy()
    bad = np.nonzero((got != want).any(1))[0]
    assert bad.size == 0, "%s: query %d differs: %s vs %s" % (label, bad[0], got[bad[0]], want[bad[0]])
    assert ev == wev, "%s: %d evaluations, oracle %d" % (label, ev, wev)
    # distances of the results: exact delta(q, id), recomputed here in float64
    bits = dist.cpu().numpy().view(np.uint32)
    Xf, Qf = X.astype(np.float64), Q.astype(np.float64)
    for q in range(0, Q.shape[0], max(1, Q.shape[0] // 25)):
        valid = got[q] >= 0
        ref = ((Xf[got[q][valid]] - Qf[q]) ** 2).sum(1)
        if X.dtype == np.uint8:
            assert (bits[q][valid] == ref.astype(np.uint32)).all()
        else:
            assert (bits[q][valid].view(np.float32) == ref.astype(np.float32)).all()
        assert (bits[q][~valid] == 0xFFFFFFFF).all()
        key = list(zip(bits[q][valid].tolist(), got[q][valid].tolist()))
        assert key == sorted(key)


@pytest.mark.parametrize("L,K,k", [(16, 32, 10), (64, 32, 10), (64, 8, 1), (128, 32, 10), (100, 200, 100),
                                   (33, 17, 33)])
def test_search_cfg1(rn, oracle_mod, L, K, k):
    c = wl.CONFIGS["cfg1"]
    X = wl.make_data(c)
    Q = wl.make_queries(c, 100)
    graph, degree = built(rn, X, c.S, c.R, c.T1, c.T2)
    check(rn, oracle_mod, X, graph, degree, Q, L, K, k, 7, "cfg1 L%d K%d k%d" % (L, K, k))


@pytest.mark.parametrize("kind,N,d", [("unit_f32", 3000, 96), ("beta_f32", 1500, 960), ("gauss_u8", 4000, 20),
                                      ("heavy_u8", 6000, 128)])
def test_search_other_data(rn, oracle_mod, kind, N, d):
    X = wl.custom(kind, N, d, 99)
    Q = wl.custom(kind, 77, d, 100)      # 77 queries: not a multiple of anything in the launch
    graph, degree = built(rn, X, 10, 48, 2, 5)
    for L, K in ((32, 16), (128, 48)):
        check(rn, oracle_mod, X, graph, degree, Q, L, K, 10, 12345, "%s L%d K%d" % (kind, L, K))


def test_search_tiny_and_degenerate(rn, oracle_mod):
    import torch
    # fewer vertices than L: the start set is every vertex
    X = wl.custom("gauss_u8", 40, 32, 5)
    Q = wl.custom("gauss_u8", 9, 32, 6)
    graph, degree = built(rn, X, 4, 8, 1, 3)
    check(rn, oracle_mod, X, graph, degree, Q, 64, 8, 10, 3, "tiny")
    # a graph with no edges at all: the result is the best of the random start set
    g0 = torch.full((40, 8), -1, dtype=torch.int32, device="cuda")
    d0 = torch.zeros(40, dtype=torch.int32, device="cuda")
    check(rn, oracle_mod, X, g0, d0, Q, 16, 8, 5, 3, "no edges")
    # no queries
    ids, _, ev = rn.rnnd_search(cuda(X), graph, degree, cuda(Q[:0].copy()), 16, 8, 5, 3)
    assert ids.shape == (0, 5) and ev == 0


def test_search_argument_errors(rn):
    X = cuda(wl.custom("gauss_u8", 40, 32, 5))
    import torch
    g = torch.zeros((40, 8), dtype=torch.int32, device="cuda")
    dg = torch.zeros(40, dtype=torch.int32, device="cuda")
    for L, K, k in ((0, 8, 1), (129, 8, 1), (16, 0, 1), (16, 8, 0), (16, 8, 17)):
        with pytest.raises(rn.RnndError) as e:
            rn.rnnd_search(X, g, dg, X[:3].contiguous(), L, K, k, 1)
        assert e.value.status == -3


def test_search_recall_cfg2(rn, oracle_mod):
    """Search quality of the GPU-built graph by the GPU search: recall@10 against exact brute force
    (CPU oracle), and identical to what the oracle's search finds on the same graph."""
    c = wl.CONFIGS["cfg2"]
    X = wl.make_data(c)
    Q = wl.make_queries(c, 200)
    graph, degree = built(rn, X, c.S, c.R, c.T1, c.T2)
    check(rn, oracle_mod, X, graph, degree, Q, 64, 32, 10, 7, "cfg2")
    ids, _, _ = rn.rnnd_search(cuda(X), graph, degree, cuda(Q), 64, 32, 10, 7)
    truth = oracle_mod.bruteforce_knn(X, Q, 10)
    assert oracle_mod.recall_at_k(ids.cpu().numpy(), truth) > 0.9
