"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  uint8 data: adjacency, distances, flags, degrees and evaluation counts bit-identical.
float data: distances are double-accumulated and rounded once on both sides, so the same
bit-exact comparison is applied (the stated tolerance -- 1e-5 relative, >= 99 % edges -- is the
fallback bar and is checked too).
"""
import os

import numpy as np
import pytest

import workloads as wl
from conftest import live
from gpu_util import assert_snapshot_equal, device_to_arrays, dist_bits_of, snapshot_to_device

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
    """0 = automatic choice (matrix-core Gram kernels where they apply), 1 = generic kernel, 2 = automatic
    with the float matrix-core scan in double precision throughout (no single-precision first pass)."""
    rn.rnnd_set_kernel_variant(request.param)
    yield request.param
    rn.rnnd_set_kernel_variant(0)


def skip_if_nothing_new(variant, X):
    """Variants 1 and 2 only differ from the automatic choice where a matrix-core kernel applies."""
    if variant == 1 and not mfma_applies(X):
        pytest.skip("automatic choice already is the generic kernel")
    if variant == 2 and mfma_applies(X) != 3:
        pytest.skip("the double-precision form only exists for the float matrix-core scan")


def mfma_applies(X):
    """Which matrix-core scan kernel the automatic choice takes for X (0: none, generic kernel)."""
    if X.dtype == np.uint8 and X.shape[1] in (32, 64, 128):
        return 2
    if X.dtype == np.float32 and X.shape[1] % 16 == 0:
        return 3
    return 0


def cuda(X):
    import torch
    return torch.from_numpy(X).cuda()


def gauss_f32(n, d, seed):
    return np.random.default_rng(seed).normal(size=(n, d)).astype(np.float32)


def clustered_u8(n, d, seed, k=8, spread=6):
    g = np.random.default_rng(seed)
    c = g.integers(20, 236, size=(k, d))
    x = c[g.integers(0, k, size=n)] + g.integers(-spread, spread + 1, size=(n, d))
    return np.clip(x, 0, 255).astype(np.uint8)


DATASETS = {
    "cfg1": lambda: wl.make_data(wl.CONFIGS["cfg1"]),
    "u8_d64_dense": lambda: clustered_u8(900, 64, 12, k=3, spread=9),   # three tight clusters: long lists
    "u8_d128": lambda: wl.custom("heavy_u8", 3000, 128, 7),
    "u8_d33_ties": lambda: clustered_u8(1500, 33, 3),          # odd d: element-wise path; many ties
    "u8_dups": lambda: np.repeat(clustered_u8(300, 16, 4), 4, axis=0),   # exact duplicates, delta = 0
    "f32_d96": lambda: wl.custom("unit_f32", 3000, 96, 9),
    "f32_d32_dense": lambda: (clustered_u8(900, 32, 13, k=3, spread=9).astype(np.float32) / 7.0),   # long lists, ties
    "f32_d960": lambda: wl.custom("beta_f32", 1200, 960, 11),
    "f32_d7": lambda: gauss_f32(1000, 7, 5),
    # quarter-integer lattice: exact ties in bulk, far more undecided pairs per vertex than the
    # single-precision pass resolves itself, so its vertices go through the double-precision second pass
    "f32_d16_lattice": lambda: (np.random.default_rng(17).integers(-2, 3, size=(2000, 16)) * 0.25).astype(np.float32),
}


@pytest.mark.parametrize("name,S,R", [("cfg1", 10, 32), ("u8_d128", 20, 96), ("u8_d33_ties", 5, 16),
                                      ("f32_d96", 20, 96), ("f32_d960", 8, 24), ("f32_d7", 128, 128),
                                      ("u8_dups", 12, 12)])
def test_random_graph(rn, oracle_mod, name, S, R):
    X = DATASETS[name]()
    want = oracle_mod.random_graph(X, S, 2310, R)
    keys, deg = rn.rnnd_random_graph(cuda(X), S, R, 2310)
    assert_snapshot_equal(want, X.dtype == np.float32, keys, deg, name)


@pytest.mark.parametrize("name,S,R", [("cfg1", 10, 32), ("u8_d128", 20, 96), ("u8_d33_ties", 6, 16),
                                      ("u8_dups", 8, 12), ("f32_d96", 20, 96), ("f32_d960", 8, 24),
                                      ("f32_d7", 100, 128), ("u8_d64_dense", 100, 128), ("u8_d128", 70, 70),
                                      ("f32_d32_dense", 90, 96), ("f32_d32_dense", 100, 128),
                                      ("f32_d16_lattice", 60, 96)])
def test_rounds_from_shared_snapshots(rn, oracle_mod, variant, name, S, R):
    """Every step starts from the oracle's snapshot, so one divergence cannot hide the next."""
    X = DATASETS[name]()
    skip_if_nothing_new(variant, X)
    isf = X.dtype == np.float32
    Xd = cuda(X)
    snap = oracle_mod.random_graph(X, S, 99, R)
    for step in ["u", "u", "u", "r", "u", "u", "r", "u"]:
        keys, deg = snapshot_to_device(snap, isf, R)
        if step == "u":
            snap, evals, props = oracle_mod.update_neighbors_sync(X, snap, R)
            st = rn.rnnd_update_neighbors(Xd, keys, deg, R, 1)
            assert st.kernel_variant == (mfma_applies(X) if variant != 1 and mfma_applies(X) else 1)
            assert st.algo_evals[0] == evals and st.proposals[0] == props
        else:
            snap = oracle_mod.add_reverse_edges(snap, R)
            rn.rnnd_add_reverse_edges(keys, deg, R)
        assert_snapshot_equal(snap, isf, keys, deg, "%s step %s" % (name, step))


@pytest.mark.parametrize("name,S,R,T1,T2", [
    ("cfg1", 10, 32, 2, 4), ("u8_d128", 20, 96, 3, 5), ("u8_d33_ties", 6, 16, 3, 4),
    ("u8_dups", 8, 12, 3, 4), ("u8_d64_dense", 40, 128, 3, 4), ("u8_d128", 60, 64, 2, 3),
    ("f32_d96", 20, 96, 3, 5), ("f32_d960", 8, 24, 2, 4), ("f32_d7", 16, 128, 2, 6),
    ("f32_d32_dense", 40, 96, 3, 4), ("f32_d32_dense", 40, 128, 2, 3), ("f32_d16_lattice", 30, 96, 2, 3)])
def test_full_build(rn, oracle_mod, variant, name, S, R, T1, T2):
    X = DATASETS[name]()
    skip_if_nothing_new(variant, X)
    isf = X.dtype == np.float32
    want = oracle_mod.build_sync(X, S, R, T1, T2, wl.BUILD_SEED)
    graph, degree, keys, st = rn.rnnd_build_ex(cuda(X), S, R, T1, T2, wl.BUILD_SEED)
    assert_snapshot_equal(want.snap, isf, keys, degree, name)
    assert (graph.cpu().numpy() == want.snap.ids).all()
    assert st.rounds == T1 * T2 and st.init_evals == len(X) * S
    assert list(st.algo_evals[:T1 * T2]) == want.round_evals.tolist()
    assert list(st.proposals[:T1 * T2]) == want.round_props.tolist()
    g2, d2 = rn.rnnd_build(cuda(X), S, R, T1, T2, wl.BUILD_SEED)      # plain entry point, and determinism
    assert (g2 == graph).all() and (d2 == degree).all()


def test_float_tolerance_bar(rn, oracle_mod, variant):
    """The stated float bar, independent of bit-exactness: delta within 1e-5 relative of a float64
    numpy evaluation, >= 99 % of edges equal to the oracle's."""
    X = DATASETS["f32_d96"]()
    want = oracle_mod.build_sync(X, 20, 48, 2, 5, 1)
    graph, degree, keys, _ = rn.rnnd_build_ex(cuda(X), 20, 48, 2, 5, 1)
    ids, bits, _, deg = device_to_arrays(keys, degree)
    Xd = X.astype(np.float64)
    edges = eq = 0
    for u in range(0, len(X), 7):
        m = deg[u]
        ref = ((Xd[ids[u, :m]] - Xd[u]) ** 2).sum(1)
        got = bits[u, :m].view(np.float32).astype(np.float64)
        assert np.all(np.abs(got - ref) <= 1e-5 * ref)
        mo = want.snap.deg[u]
        edges += max(m, mo)
        eq += len(set(ids[u, :m].tolist()) & set(want.snap.ids[u, :mo].tolist()))
    assert eq >= 0.99 * edges


def test_hub_vertex_streams_through_the_merge(rn, oracle_mod, variant):
    """A star: vertex 0 sits at the centre of everything, so hundreds of edges are redirected to
    it in one round and hundreds of reverse edges enter it (the > 128-key path of the merge and
    the in-degree cap of Alg. 5)."""
    if variant == 2:
        pytest.skip("uint8 data: variant 2 is the automatic choice")
    g = np.random.default_rng(8)
    n, d, R = 2500, 32, 16
    X = np.clip(128 + g.normal(0, 40, size=(n, d)), 0, 255).astype(np.uint8)
    X[0] = 128
    snap = oracle_mod.random_graph(X, 8, 5, R)
    for u in range(1, n):                      # plant 0 in every list
        if 0 not in snap.ids[u, :snap.deg[u]]:
            k = snap.deg[u] - 1
            snap.ids[u, k] = 0
            snap.dist[u, k] = float(((X[u].astype(np.int64) - 128) ** 2).sum())
        m = snap.deg[u]
        order = np.lexsort((snap.ids[u, :m], snap.dist[u, :m]))
        snap.ids[u, :m], snap.dist[u, :m] = snap.ids[u, :m][order], snap.dist[u, :m][order]
    Xd = cuda(X)
    for step in ["u", "r", "u", "u", "r", "u"]:
        keys, deg = snapshot_to_device(snap, False, R)
        if step == "u":
            snap, evals, props = oracle_mod.update_neighbors_sync(X, snap, R)
            st = rn.rnnd_update_neighbors(Xd, keys, deg, R, 1)
            assert st.algo_evals[0] == evals and st.proposals[0] == props
        else:
            snap = oracle_mod.add_reverse_edges(snap, R)
            rn.rnnd_add_reverse_edges(keys, deg, R)
        assert_snapshot_equal(snap, False, keys, deg, "hub step " + step)


def test_tiny_and_degenerate_inputs(rn, oracle_mod, variant):
    if variant == 2:
        pytest.skip("uint8 data: variant 2 is the automatic choice")
    # N = 2: the only possible graph
    X = np.array([[0, 0], [3, 4]], np.uint8)
    g, d = rn.rnnd_build(cuda(X), 1, 1, 2, 2, 0)
    assert g.cpu().numpy().tolist() == [[1], [0]] and d.cpu().numpy().tolist() == [1, 1]
    # all points identical: every delta is 0, every test ties, order is by id alone
    X = np.full((40, 32), 7, np.uint8)
    want = oracle_mod.build_sync(X, 5, 8, 2, 3, 4)
    graph, degree, keys, _ = rn.rnnd_build_ex(cuda(X), 5, 8, 2, 3, 4)
    assert_snapshot_equal(want.snap, False, keys, degree, "identical points")
    # complete initialisation, R = RNND_MAX_R
    X = clustered_u8(129, 32, 6)
    want = oracle_mod.build_sync(X, 128, 128, 2, 3, 4)
    graph, degree, keys, _ = rn.rnnd_build_ex(cuda(X), 128, 128, 2, 3, 4)
    assert_snapshot_equal(want.snap, False, keys, degree, "complete init")
    # a snapshot with empty rows and no "new" entry at all: nothing may change
    snap = oracle_mod.Snapshot.empty(50, 8)
    X = clustered_u8(50, 32, 7)
    keys, deg = snapshot_to_device(snap, False, 8)
    st = rn.rnnd_update_neighbors(cuda(X), keys, deg, 8, 2)
    assert st.active[0] == 0 and (deg == 0).all()
    rn.rnnd_add_reverse_edges(keys, deg, 8)
    assert (deg == 0).all()


def test_argument_errors_on_device(rn):
    import torch
    X = torch.zeros((10, 16), dtype=torch.uint8, device="cuda")
    for kw, status in [(dict(S=0, R=4), -3), (dict(S=5, R=4), -3), (dict(S=2, R=129), -3),
                       (dict(S=10, R=12), -3)]:
        with pytest.raises(rn.RnndError) as e:
            rn.rnnd_build(X, kw["S"], kw["R"], 1, 1, 0)
        assert e.value.status == status
    with pytest.raises(rn.RnndError) as e:
        rn.rnnd_build(X, 2, 4, 1, 1, 0, metric=3)
    assert e.value.status == -4
    with pytest.raises(rn.RnndError) as e:
        rn.rnnd_build(X[:1].contiguous(), 1, 4, 1, 1, 0)
    assert e.value.status == -2


def test_cfg2_full_parity(rn, oracle_mod, variant):
    """Workload cfg2 (N = 100,000, d = 128 uint8, paper parameters): ~20 s of oracle."""
    if variant == 2:
        pytest.skip("uint8 data: variant 2 is the automatic choice")
    c = wl.CONFIGS["cfg2"]
    X = wl.make_data(c)
    want = oracle_mod.build_sync(X, c.S, c.R, c.T1, c.T2, wl.BUILD_SEED)
    graph, degree, keys, st = rn.rnnd_build_ex(cuda(X), c.S, c.R, c.T1, c.T2, wl.BUILD_SEED)
    assert_snapshot_equal(want.snap, False, keys, degree, "cfg2")
    assert list(st.algo_evals[:60]) == want.round_evals.tolist()
    # the plain entry point (no statistics, no timing events) builds the same graph
    g1, d1 = rn.rnnd_build(cuda(X), c.S, c.R, c.T1, c.T2, wl.BUILD_SEED)
    assert (g1 == graph).all() and (d1 == degree).all()
    assert (g1.cpu().numpy() == want.snap.ids).all()


@pytest.mark.slow
@live
def test_cfg3_full_size_parity(rn, oracle_mod):
    """Workload cfg3 -- the benchmark's workload (N = 1,000,000, d = 128 uint8, S=20 R=96
    T1=4 T2=15) in the launch configuration bench.py times: the whole graph, every distance, flag,
    degree and per-round evaluation count against a full oracle run (about a minute of CPU)."""
    import time
    c = wl.CONFIGS["cfg3"]
    X = wl.make_data(c)
    print("cfg3 data ready", wl.sha256_of(X)[:16], flush=True)
    graph, degree, keys, st = rn.rnnd_build_ex(cuda(X), c.S, c.R, c.T1, c.T2, wl.BUILD_SEED)
    print("gpu build done: %.1f ms" % st.total_ms, flush=True)
    t0 = time.time()
    want = oracle_mod.build_sync(X, c.S, c.R, c.T1, c.T2, wl.BUILD_SEED, progress=True)
    print("oracle build done: %.1f s" % (time.time() - t0), flush=True)
    assert_snapshot_equal(want.snap, False, keys, degree, "cfg3")
    assert (graph.cpu().numpy() == want.snap.ids).all()
    assert list(st.algo_evals[:60]) == want.round_evals.tolist()
    assert list(st.proposals[:60]) == want.round_props.tolist()
    # search on the full-size graph: GPU search against the oracle's, 300 of the configuration's queries
    Q = wl.make_queries(c, 300)
    for L, K in ((64, 32), (128, 96)):
        found, _, evals = rn.rnnd_search(cuda(X), graph, degree, cuda(Q), L, K, 10, 7)
        wfound, wevals = oracle_mod.search(X, want.snap.ids, want.snap.deg, Q, L, K, 10, 7)
        assert (found.cpu().numpy() == wfound).all() and evals == wevals
        print("search parity ok: L %d K %d, %.0f evaluations per query" % (L, K, evals / 300), flush=True)


FULL = os.environ.get("RNND_FULL_PARITY", "") == "1"


@pytest.mark.slow
@pytest.mark.skipif(not FULL, reason="set RNND_FULL_PARITY=1: several minutes of single-threaded oracle")
@live
def test_cfg4_full_size_parity(rn, oracle_mod):
    """Workload cfg4 (N = 1,000,000, d = 96 float32, unit vectors) against a full oracle run."""
    import time
    c = wl.CONFIGS["cfg4"]
    X = wl.make_data(c)
    print("cfg4 data ready", wl.sha256_of(X)[:16], flush=True)
    graph, degree, keys, st = rn.rnnd_build_ex(cuda(X), c.S, c.R, c.T1, c.T2, wl.BUILD_SEED)
    print("gpu build done: %.1f ms" % st.total_ms, flush=True)
    t0 = time.time()
    want = oracle_mod.build_sync(X, c.S, c.R, c.T1, c.T2, wl.BUILD_SEED, progress=True)
    print("oracle build done: %.1f s" % (time.time() - t0), flush=True)
    ids, bits, flags, deg = device_to_arrays(keys, degree)
    rows_equal = ((ids == want.snap.ids).all(1) & (deg == want.snap.deg)).mean()
    print("rows identical: %.6f" % rows_equal, flush=True)
    assert_snapshot_equal(want.snap, True, keys, degree, "cfg4")
    assert list(st.algo_evals[:60]) == want.round_evals.tolist()


def _full_size_sampled_parity(rn, oracle_mod, name, half=False):
    """A float workload at full size in the launch configuration bench.py times.  A full oracle run takes
    minutes (cfg4) to hours (cfg5), so outputs are sampled: after the GPU has run RandomGraph
    and k rounds, one more round is run on the GPU, and for 2,000 sampled vertices the oracle computes
    that round one vertex at a time (a snapshot in which only the sampled lists are non-empty).  The
    entries the GPU kept for a sampled vertex (flag old) must equal the oracle's kept list, key for key
    (up to the cut at R when the full graph redirected more edges to it than the sample can know);
    RandomGraph rows of the sample are compared the same way; structure (sorted, distinct, no self loop,
    degree <= R, distances = float64 numpy) is checked on the sample of the final graph."""
    c = wl.CONFIGS[name]
    X = wl.make_data(c)
    print("%s data ready" % name, flush=True)
    if half:        # half-precision storage: the expected graph is the oracle's on the floats the halves stand for
        X16 = X.astype(np.float16)
        X = X16.astype(np.float32)
        Xd = cuda(X16)
    else:
        Xd = cuda(X)
    R = c.R
    g = np.random.default_rng(1)
    sample = np.sort(g.choice(c.N, 2000, replace=False))
    keys, deg = rn.rnnd_random_graph(Xd, c.S, R, wl.BUILD_SEED)
    ids0, bits0, flags0, deg0 = device_to_arrays(keys, deg)
    for u in sample[:300]:
        want_ids = oracle_mod.random_ids(c.N, int(u), c.S, wl.BUILD_SEED)
        assert sorted(ids0[u, :c.S].tolist()) == sorted(want_ids.tolist())
    for k_before in (0, 3):
        if k_before:
            rn.rnnd_update_neighbors(Xd, keys, deg, R, k_before)
        ids_b, bits_b, flags_b, deg_b = device_to_arrays(keys, deg)
        snap = oracle_mod.Snapshot.empty(c.N, R)
        for u in sample:
            m = deg_b[u]
            snap.ids[u, :m] = ids_b[u, :m]
            snap.dist[u, :m] = bits_b[u, :m].view(np.float32).astype(np.float64)
            snap.flags[u, :m] = flags_b[u, :m]
            snap.deg[u] = m
        want, _, _ = oracle_mod.update_neighbors_sync(X, snap, R)
        rn.rnnd_update_neighbors(Xd, keys, deg, R, 1)
        ids_a, bits_a, flags_a, deg_a = device_to_arrays(keys, deg)
        sampled = set(sample.tolist())
        for u in sample:
            got = [(int(bits_a[u, k]), int(ids_a[u, k])) for k in range(deg_a[u]) if flags_a[u, k] == 0]
            # in the reduced snapshot nothing is redirected INTO u unless its source is sampled too
            wk = [(int(np.float32(want.dist[u, k]).view(np.uint32)), int(want.ids[u, k]))
                  for k in range(want.deg[u]) if want.flags[u, k] == 0]
            if deg_a[u] < R:
                assert got == wk, "vertex %d after %d rounds" % (u, k_before)
            else:
                # a full row: edges redirected to u by vertices outside the sample may have pushed the
                # farthest kept entries past the cut at R; what is missing must lie beyond the last key
                last = (int(bits_a[u, R - 1]), int(ids_a[u, R - 1]))
                assert set(got) <= set(wk) and all(k > last for k in set(wk) - set(got)), "vertex %d" % u
        print("sampled round parity ok after %d rounds" % k_before, flush=True)
    graph, degree, fkeys, st = rn.rnnd_build_ex(Xd, c.S, R, c.T1, c.T2, wl.BUILD_SEED)
    print("gpu build done: %.1f ms" % st.total_ms, flush=True)
    ids, bits, flags, dg = device_to_arrays(fkeys, degree)
    Xs = X.astype(np.float64)
    for u in sample[:500]:
        m = dg[u]
        row = ids[u, :m]
        assert m <= R and len(set(row.tolist())) == m and u not in row
        ref = ((Xs[row] - Xs[u]) ** 2).sum(1).astype(np.float32)
        assert (bits[u, :m].view(np.float32) == ref).all()
        key = list(zip(bits[u, :m].tolist(), row.tolist()))
        assert key == sorted(key)


@pytest.mark.slow
@live
def test_cfg5_full_size_sampled_parity(rn, oracle_mod):
    """Workload cfg5 (N = 1,000,000, d = 960 float32)."""
    _full_size_sampled_parity(rn, oracle_mod, "cfg5")


@pytest.mark.slow
@live
def test_cfg4_full_size_sampled_parity(rn, oracle_mod):
    """Workload cfg4 (N = 1,000,000, d = 96 float32, unit vectors); the full oracle run is
    test_cfg4_full_size_parity."""
    _full_size_sampled_parity(rn, oracle_mod, "cfg4")


@pytest.mark.slow
@live
def test_cfg4_full_size_sampled_parity_half_storage(rn, oracle_mod):
    """The same with the rows handed over in half precision (the f16 matrix-instruction path of the scan)."""
    _full_size_sampled_parity(rn, oracle_mod, "cfg4", half=True)


@pytest.mark.slow
@live
def test_cfg5_full_size_sampled_parity_half_storage(rn, oracle_mod):
    """Workload cfg5 (rows of 960 coordinates) in half precision."""
    _full_size_sampled_parity(rn, oracle_mod, "cfg5", half=True)


def test_gather_probe_reports_a_plausible_rate(rn):
    """The measurement aid behind the 'gather ceiling' of the benchmark line: it must run on rows of any
    multiple of 16 bytes and report something between a trickle and the HBM peak times the cache effect."""
    import torch
    for rows, width, dtype in ((200_000, 128, torch.uint8), (50_000, 96, torch.float32), (3_000, 48, torch.uint8),
                               (1, 16, torch.uint8)):
        X = torch.zeros((rows, width), dtype=dtype, device="cuda")
        rate = rn.rnnd_probe_gather(X, 2_000_000)
        assert 1.0 < rate < 100_000.0, (rows, width, rate)


def test_build_on_a_side_stream_and_repeated_calls(rn):
    """All work goes to the stream handed in (default priority) and the call returns after it has completed;
    the result does not depend on the stream, and repeated calls leave nothing behind that changes it."""
    import torch
    c = wl.CONFIGS["cfg1"]
    X = cuda(wl.make_data(c))
    g0, d0 = rn.rnnd_build(X, c.S, c.R, c.T1, c.T2, wl.BUILD_SEED)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        g1, d1 = rn.rnnd_build(X, c.S, c.R, c.T1, c.T2, wl.BUILD_SEED)
        ids1, _, _ = rn.rnnd_search(X, g1, d1, X[:50].contiguous(), 32, 32, 5, 3)
    side.synchronize()
    ids0, _, _ = rn.rnnd_search(X, g0, d0, X[:50].contiguous(), 32, 32, 5, 3)
    assert (g0 == g1).all() and (d0 == d1).all() and (ids0 == ids1).all()
    for _ in range(5):
        g2, d2 = rn.rnnd_build(X, c.S, c.R, c.T1, c.T2, wl.BUILD_SEED)
    assert (g0 == g2).all() and (d0 == d2).all()
    assert (ids0[:, 0].cpu() == torch.arange(50, dtype=torch.int32)).all()     # a point's nearest neighbour is itself
