"""16-bit storage (RNND_F16: IEEE half, RNND_BF16: bfloat16): every coordinate stands for the float32 value it
converts to exactly, so the expected graph is the oracle's on the widened matrix -- ids, distances (float32
bits), flags, degrees, evaluation counts; search likewise."""
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


@pytest.fixture(params=[0, 1, 2], ids=["auto", "generic", "f64"])
def variant(request, rn):
    rn.rnnd_set_kernel_variant(request.param)
    yield request.param
    rn.rnnd_set_kernel_variant(0)


def cuda(a):
    import torch
    return torch.from_numpy(a).cuda()


def _half(kind, n, d, seed):
    if kind == "unit":
        x = wl.custom("unit_f32", n, d, seed)
    elif kind == "beta":
        x = wl.custom("beta_f32", n, d, seed)
    elif kind == "lattice":
        x = (np.random.default_rng(seed).integers(-2, 3, size=(n, d)) * 0.25).astype(np.float32)
    else:
        x = np.random.default_rng(seed).normal(size=(n, d)).astype(np.float32)
    return x.astype(np.float16)


CASES = [
    # kind, N, d, S, R, T1, T2
    ("unit", 3000, 96, 20, 96, 3, 4),
    ("beta", 1200, 960, 8, 24, 2, 4),
    ("gauss", 1000, 7, 16, 128, 2, 5),
    ("gauss", 2000, 40, 10, 33, 2, 4),       # rows of 80 bytes: 16-byte chunks, no matrix-core path
    ("gauss", 1500, 64, 12, 48, 2, 4),
    ("lattice", 2000, 32, 30, 96, 2, 3),
    ("gauss", 900, 12, 5, 9, 2, 3),          # rows of 24 bytes: element-wise path
    ("unit", 2500, 160, 40, 128, 2, 3),
    ("gauss", 2, 32, 1, 1, 1, 2),
]


@pytest.mark.parametrize("kind,N,d,S,R,T1,T2", CASES)
def test_build_on_half_rows(rn, oracle_mod, variant, kind, N, d, S, R, T1, T2):
    if variant == 2 and d % 32 != 0:
        pytest.skip("no matrix-core scan for this row length")
    X16 = _half(kind, N, d, 300 + N + d)
    X = X16.astype(np.float32)                       # exact
    want = oracle_mod.build_sync(X, S, R, T1, T2, 21)
    graph, degree, keys, st = rn.rnnd_build_ex(cuda(X16), S, R, T1, T2, 21)
    assert_snapshot_equal(want.snap, True, keys, degree, "%s N %d d %d" % (kind, N, d))
    assert (graph.cpu().numpy() == want.snap.ids).all()
    assert list(st.algo_evals[:T1 * T2]) == want.round_evals.tolist()
    assert list(st.proposals[:T1 * T2]) == want.round_props.tolist()
    # the float32 build of the widened matrix gives the same graph
    g32, d32 = rn.rnnd_build(cuda(X), S, R, T1, T2, 21)
    assert (g32 == graph).all() and (d32 == degree).all()
    # search
    Q16 = _half(kind, 9, d, 7)
    for L, K in ((16, 8), (100, 200)):
        found, bits, evals = rn.rnnd_search(cuda(X16), graph, degree, cuda(Q16), L, K, min(10, L), 3, want_dist=True)
        wfound, wevals = oracle_mod.search(X, want.snap.ids, want.snap.deg, Q16.astype(np.float32), L, K, min(10, L), 3)
        assert (found.cpu().numpy() == wfound).all() and evals == wevals


def test_blocks_and_steps_on_half_rows(rn, oracle_mod):
    X16 = _half("unit", 1500, 96, 5)
    X = X16.astype(np.float32)
    want = oracle_mod.build_blocks(X, 10, 40, 2, 3, 4, 6)
    graph, degree, keys, _ = rn.rnnd_build_blocks(cuda(X16), 10, 40, 2, 3, 4, 6)
    assert_snapshot_equal(want.snap, True, keys, degree, "half rows, 6 runs per pass")
    k2, d2 = rn.rnnd_random_graph(cuda(X16), 10, 40, 4)
    snap = oracle_mod.random_graph(X, 10, 4, 40)
    assert_snapshot_equal(snap, True, k2, d2, "half rows, RandomGraph")
    snap, evals, props = oracle_mod.update_neighbors_sync(X, snap, 40)
    st = rn.rnnd_update_neighbors(cuda(X16), k2, d2, 40, 1)
    assert_snapshot_equal(snap, True, k2, d2, "half rows, one round")
    assert st.algo_evals[0] == evals and st.proposals[0] == props


BF_CASES = [
    ("unit", 3000, 96, 20, 96, 2, 4),
    ("beta", 1000, 960, 8, 24, 2, 3),
    ("gauss", 1500, 40, 10, 33, 2, 3),
    ("gauss", 900, 12, 5, 9, 2, 3),
    ("lattice", 1500, 32, 30, 96, 2, 2),
    ("unit", 2000, 160, 40, 128, 2, 2),
]


@pytest.mark.parametrize("kind,N,d,S,R,T1,T2", BF_CASES)
def test_build_on_bfloat16_rows(rn, oracle_mod, variant, kind, N, d, S, R, T1, T2):
    import torch
    if variant == 2 and d % 32 != 0:
        pytest.skip("no matrix-core scan for this row length")
    Xb = torch.from_numpy(_half(kind, N, d, 500 + N + d).astype(np.float32)).to(torch.bfloat16).cuda()
    X = Xb.float().cpu().numpy()                    # exact widening
    want = oracle_mod.build_sync(X, S, R, T1, T2, 22)
    graph, degree, keys, st = rn.rnnd_build_ex(Xb, S, R, T1, T2, 22)
    assert_snapshot_equal(want.snap, True, keys, degree, "bf16 %s N %d d %d" % (kind, N, d))
    assert list(st.algo_evals[:T1 * T2]) == want.round_evals.tolist()
    Qb = torch.from_numpy(_half(kind, 9, d, 8).astype(np.float32)).to(torch.bfloat16).cuda()
    found, _, evals = rn.rnnd_search(Xb, graph, degree, Qb, 32, 16, 10, 3)
    wfound, wevals = oracle_mod.search(X, want.snap.ids, want.snap.deg, Qb.float().cpu().numpy(), 32, 16, 10, 3)
    assert (found.cpu().numpy() == wfound).all() and evals == wevals
