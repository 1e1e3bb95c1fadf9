"""Pins for the CPU oracle: each test checks it against something the paper or the
mathematics fixes, never against itself.  (CPU only.)

  Fig. 1(c) worked example, tie rule         -> Alg. 4 (prune test, redirect)
  reduction to Alg. 3 / exact RNG / 1-NN     -> Sec. 4.2 (Alg. 4 is Alg. 3 applied to the current neighbours)
  path-graph fixed point on a 1-D lattice    -> Alg. 4 (closed form)
  Eq. 2 on kept neighbours, degree bounds    -> Eq. 2, Alg. 5, Sec. 5.3
  flag skip changes cost, not results        -> Sec. 4.2 last paragraph
  set-wise brute-force models on tiny inputs -> Alg. 4, Alg. 5 written a second way
  block-sequential passes: worked example of the vertex order, one block = synchronous round,
  n blocks = the in-place order of Alg. 4's vertex loop  -> Alg. 4
"""
import numpy as np
import pytest

import workloads as wl
from conftest import read_golden, snapshot_from_lists

M64 = 2**64 - 1


# ----------------------------------------------------------------- helpers
def sqdist_matrix(X):
    """All-pairs squared L2 by numpy; float data rounded once from float64 like the oracle states."""
    Xd = X.astype(np.float64)
    D = ((Xd[:, None, :] - Xd[None, :, :]) ** 2).sum(-1)
    if X.dtype == np.float32:
        D = D.astype(np.float32).astype(np.float64)
    return D


def rows_of(snap, u):
    m = int(snap.deg[u])
    return [(float(snap.dist[u, k]), int(snap.ids[u, k]), int(snap.flags[u, k])) for k in range(m)]


def small_u8(n, d, seed, lo=0, hi=256):
    return np.random.default_rng(seed).integers(lo, hi, size=(n, d)).astype(np.uint8)


def small_f32(n, d, seed):
    return np.random.default_rng(seed).normal(size=(n, d)).astype(np.float32)


# ------------------------------------------------- RandomGraph (Alg. 6)
def test_mix64_matches_published_splitmix64_vector(oracle_mod):
    vec = [int(line) for line in open(__import__("os").path.join(
        __import__("conftest").GOLDEN, "splitmix64_seed1234567.txt")) if line[0].isdigit()]
    x = 1234567
    for want in vec:
        x = (x + 0x9E3779B97F4A7C15) & M64
        assert oracle_mod.mix64(x) == want


def test_draw_is_two_nested_mix64_calls(oracle_mod):
    """draw j of vertex u = mix64(mix64(seed + G (u + 1)) + G (j + 1)), recomputed here from mix64 alone (which
    the published vector above pins): a swapped u and j, a missing + 1 or a single mix would all differ."""
    G = 0x9E3779B97F4A7C15
    for seed, u, j in [(0, 0, 0), (2310, 5, 0), (2310, 0, 5), (99, 123456, 77), (M64, 2**31 - 2, 1023)]:
        inner = oracle_mod.mix64((seed + G * (u + 1)) & M64)
        assert oracle_mod.draw(seed, u, j) == oracle_mod.mix64((inner + G * (j + 1)) & M64)
    assert oracle_mod.draw(1, 2, 3) != oracle_mod.draw(1, 3, 2)


def test_random_ids_are_distinct_in_range_and_seeded(oracle_mod):
    n, S = 1000, 20
    seen_rows = []
    for u in [0, 1, 499, 999]:
        ids = oracle_mod.random_ids(n, u, S, 2310)
        assert len(set(ids.tolist())) == S and u not in ids
        assert ids.min() >= 0 and ids.max() < n
        assert (ids == oracle_mod.random_ids(n, u, S, 2310)).all()
        assert (ids != oracle_mod.random_ids(n, u, S, 2311)).any()
        seen_rows.append(tuple(ids.tolist()))
    assert len(set(seen_rows)) == len(seen_rows)


def test_random_ids_follow_the_stated_draw_mapping(oracle_mod):
    # id_j = c + (c >= u), c = ((draw >> 32) * (n-1)) >> 32, repeats skipped
    n, u, S, seed = 37, 5, 12, 99
    want, j = [], 0
    while len(want) < S:
        z = oracle_mod.draw(seed, u, j)
        c = ((z >> 32) * (n - 1)) >> 32
        v = c + (1 if c >= u else 0)
        if v not in want:
            want.append(v)
        j += 1
    assert oracle_mod.random_ids(n, u, S, seed).tolist() == want


def test_random_ids_cover_everything_when_S_is_n_minus_1(oracle_mod):
    n = 24
    for u in range(n):
        ids = oracle_mod.random_ids(n, u, n - 1, 5)
        assert sorted(ids.tolist()) == [v for v in range(n) if v != u]


def test_random_ids_roughly_uniform(oracle_mod):
    n, S = 50, 5
    cnt = np.zeros(n)
    for seed in range(400):
        for v in oracle_mod.random_ids(n, 7, S, seed):
            cnt[v] += 1
    assert cnt[7] == 0
    other = np.delete(cnt, 7)
    # 2000 draws over 49 bins: mean 40.8, sd ~6.3
    assert other.min() > 15 and other.max() < 70


# ------------------------------------------------------------------ Eq. 3
def test_delta_matches_numpy(oracle_mod):
    X = small_u8(40, 33, 1)
    D = sqdist_matrix(X)
    for a, b in [(0, 1), (5, 17), (39, 0), (3, 3)]:
        assert oracle_mod.delta(X, a, b) == D[a, b] == oracle_mod.delta(X, b, a)
    Xf = small_f32(40, 97, 2)
    Df = sqdist_matrix(Xf)
    for a, b in [(0, 1), (5, 17), (39, 0), (3, 3)]:
        assert oracle_mod.delta(Xf, a, b) == Df[a, b] == oracle_mod.delta(Xf, b, a)


def test_delta_u8_extremes(oracle_mod):
    X = np.zeros((2, 128), np.uint8)
    X[1] = 255
    assert oracle_mod.delta(X, 0, 1) == 128 * 255 * 255


# ------------------------------------------------- Alg. 4 worked examples
@pytest.mark.parametrize("fixture", ["fig1c_redirect.txt", "tie_prunes.txt"])
def test_worked_example(oracle_mod, fixture):
    g = read_golden(fixture)
    X = np.array(g["points"], np.uint8)
    lists = [g["initial_list_of_0"][0]] + [[] for _ in range(len(X) - 1)]
    s0 = snapshot_from_lists(oracle_mod, X, lists, 8)
    s1, evals, props = oracle_mod.update_neighbors_sync(X, s0, 8)
    assert [i for _, i, _ in rows_of(s1, 0)] == g["kept_of_0"][0]
    assert all(f == 0 for _, _, f in rows_of(s1, 0))            # kept entries become old
    r1 = rows_of(s1, 1)
    assert [i for _, i, _ in r1] == g["row_of_1_after"][0]
    assert [d for d, _, _ in r1] == [float(g["dist_of_that_entry"][0][0])]
    assert all(f == 1 for _, _, f in r1)                        # redirected entries are new
    assert evals == g["evaluations"][0][0] and props == 1
    for u in range(2, len(X)):
        assert s1.deg[u] == 0


# ------------------------------------- reduction to Alg. 3 and the exact RNG
def py_rng_strategy(D, u, cand):
    order = sorted(cand, key=lambda v: (D[u, v], v))
    kept = []
    for v in order:
        if all(D[u, v] < D[v, w] for w in kept):
            kept.append(v)
    return kept


def exact_rng_neighbours(D, u):
    n = len(D)
    return {v for v in range(n) if v != u and
            not any(max(D[u, w], D[v, w]) < D[u, v] for w in range(n) if w not in (u, v))}


@pytest.mark.parametrize("kind", ["u8", "f32"])
def test_complete_init_first_pass_is_rng_strategy(oracle_mod, kind):
    n = 40
    X = small_u8(n, 6, 11) if kind == "u8" else small_f32(n, 6, 12)
    D = sqdist_matrix(X)
    s0 = oracle_mod.random_graph(X, n - 1, 123, n)
    for u in range(n):                                          # structural: complete, sorted, exact dists
        r = rows_of(s0, u)
        assert sorted(i for _, i, _ in r) == [v for v in range(n) if v != u]
        assert r == sorted(r) and all(d == D[u, i] and f == 1 for d, i, f in r)
    s1, evals, _ = oracle_mod.update_neighbors_sync(X, s0, n)
    tri = D[np.triu_indices(n, 1)]
    distinct = len(np.unique(tri)) == len(tri)
    for u in range(n):
        kept = [i for _, i, f in rows_of(s1, u) if f == 0]
        want = py_rng_strategy(D, u, [v for v in range(n) if v != u])
        assert kept == want
        assert kept == oracle_mod.rng_strategy(X, u, np.array([v for v in range(n) if v != u])).tolist()
        nn = min((D[u, v], v) for v in range(n) if v != u)[1]
        assert kept[0] == nn                                    # exact nearest neighbour survives
        if distinct:
            assert exact_rng_neighbours(D, u) <= set(kept)      # textbook RNG is contained


def test_rng_strategy_on_a_square_with_centre(oracle_mod):
    # centre of a square: all four corners are kept (corner-corner 16 > corner-centre 8); textbook case
    X = np.array([[2, 2], [0, 0], [4, 0], [0, 4], [4, 4]], np.uint8)
    assert oracle_mod.rng_strategy(X, 0, np.array([1, 2, 3, 4])).tolist() == [1, 2, 3, 4]
    # from a corner: centre (8) kept; adjacent corners (16): delta to centre 8 <= 16 -> pruned
    assert oracle_mod.rng_strategy(X, 1, np.array([0, 2, 3, 4])).tolist() == [0]


# ------------------------------------------- 1-D lattice: path-graph fixed point
@pytest.mark.parametrize("n", [5, 9, 14])
def test_lattice_converges_to_path_graph(oracle_mod, n):
    X = np.arange(n, dtype=np.uint8).reshape(n, 1)
    res = oracle_mod.build_sync(X, n - 1, n, 1, n, 77)
    for i in range(n):
        got = sorted(i2 for _, i2, _ in rows_of(res.snap, i))
        assert got == [j for j in (i - 1, i + 1) if 0 <= j < n]
    assert res.round_evals[-1] == 0 and res.round_props[-1] == 0   # nothing left to test


# ------------------------------------------------------ invariants after builds
def check_structure(snap, D, R, n):
    for u in range(n):
        r = rows_of(snap, u)
        ids = [i for _, i, _ in r]
        assert len(ids) == len(set(ids)) <= R and u not in ids
        assert all(0 <= i < n for i in ids)
        assert [(d, i) for d, i, _ in r] == sorted((d, i) for d, i, _ in r)
        assert all(d == D[u, i] for d, i, _ in r)
        assert (snap.ids[u, len(ids):] == -1).all()


def check_rng_invariant_on_old(snap, D, n):
    """Eq. 2 for every pair of old entries (w before v): delta(u,v) < delta(v,w) and delta(u,w) < delta(v,w)."""
    for u in range(n):
        old = [(d, i) for d, i, f in rows_of(snap, u) if f == 0]
        for a in range(len(old)):
            for b in range(a):
                (dv, v), (dw, w) = old[a], old[b]
                assert dv < D[v, w] and dw < D[v, w]


def in_degrees(snap, n):
    c = np.zeros(n, np.int64)
    for u in range(n):
        for k in range(snap.deg[u]):
            c[snap.ids[u, k]] += 1
    return c


@pytest.mark.parametrize("kind,n,d,S,R,T1,T2", [
    ("u8", 300, 8, 6, 12, 3, 4), ("f32", 300, 8, 6, 12, 3, 4), ("u8", 200, 3, 10, 16, 2, 5),
    ("u8", 120, 2, 5, 5, 3, 3)])
def test_build_invariants(oracle_mod, kind, n, d, S, R, T1, T2):
    X = small_u8(n, d, 21, 0, 40) if kind == "u8" else small_f32(n, d, 22)   # small range => many ties
    D = sqdist_matrix(X)
    snap = oracle_mod.random_graph(X, S, 5, R)
    check_structure(snap, D, R, n)
    assert (snap.deg == S).all() and (snap.flags[:, :S] == 1).all()
    for t1 in range(T1):
        for t2 in range(T2):
            before = in_degrees(snap, n)
            snap, _, _ = oracle_mod.update_neighbors_sync(X, snap, R)
            check_structure(snap, D, R, n)
            check_rng_invariant_on_old(snap, D, n)
            assert (in_degrees(snap, n) <= before).all()        # a redirect never raises an in-degree
        if t1 != T1 - 1:
            snap = oracle_mod.add_reverse_edges(snap, R)
            check_structure(snap, D, R, n)
            assert in_degrees(snap, n).max() <= R and snap.deg.max() <= R
    full = oracle_mod.build_sync(X, S, R, T1, T2, 5).snap
    assert (full.ids == snap.ids).all() and (full.deg == snap.deg).all()
    assert (full.dist == snap.dist).all() and (full.flags == snap.flags).all()
    if T1 >= 2:
        assert in_degrees(full, n).max() <= R                   # Sec. 5.3: in-degree limited to R


@pytest.mark.parametrize("kind", ["u8", "f32"])
def test_flag_skip_changes_cost_not_result(oracle_mod, kind):
    X = small_u8(400, 6, 31, 0, 30) if kind == "u8" else small_f32(400, 6, 32)
    a = oracle_mod.build_sync(X, 8, 16, 3, 5, 9, use_flag_skip=True)
    b = oracle_mod.build_sync(X, 8, 16, 3, 5, 9, use_flag_skip=False)
    assert (a.snap.ids == b.snap.ids).all() and (a.snap.deg == b.snap.deg).all()
    assert (a.snap.flags == b.snap.flags).all()
    assert a.round_evals.sum() < b.round_evals.sum()
    assert a.round_evals[0] == b.round_evals[0]                 # first pass: everything is new
    assert (a.round_props == b.round_props).all()


# ------------------------------- set-wise models of Alg. 4 / Alg. 5 on tiny inputs
def py_sync_round(D, lists, R):
    """lists[u] = {id: flag}.  Alg. 4 per vertex on the snapshot, then merge; written with dicts/sets."""
    n = len(lists)
    kept = [dict() for _ in range(n)]
    incoming = [dict() for _ in range(n)]
    evals = 0
    for u in range(n):
        order = sorted(lists[u], key=lambda v: (D[u, v], v))
        sel = []
        for v in order:
            ok = True
            for w in sel:
                if lists[u][v] == 0 and lists[u][w] == 0:
                    continue
                evals += 1
                if D[u, v] >= D[v, w]:
                    incoming[w][v] = 1
                    ok = False
                    break
            if ok:
                sel.append(v)
        kept[u] = {v: 0 for v in sel}
    out = []
    for x in range(n):
        cand = dict(incoming[x])
        cand.update(kept[x])                                    # an existing entry wins
        order = sorted(cand, key=lambda v: (D[x, v], v))[:R]
        out.append({v: cand[v] for v in order})
    return out, evals


def py_add_reverse(D, lists, R):
    n = len(lists)
    E = {(u, v): f for u in range(n) for v, f in lists[u].items()}
    for (u, v) in list(E):
        if (v, u) not in E:
            E[(v, u)] = 1
    for v in range(n):                                          # edges leaving v: keep R shortest
        out = sorted((D[v, u], u) for (a, u) in E if a == v)
        for _, u in out[R:]:
            del E[(v, u)]
    for v in range(n):                                          # edges entering v: keep R shortest
        inc = sorted((D[u, v], u) for (u, b) in E if b == v)
        for _, u in inc[R:]:
            del E[(u, v)]
    res = [dict() for _ in range(n)]
    for (u, v), f in E.items():
        res[u][v] = f
    return res


def lists_of(snap, n):
    return [{int(snap.ids[u, k]): int(snap.flags[u, k]) for k in range(snap.deg[u])} for u in range(n)]


@pytest.mark.parametrize("seed,R", [(1, 4), (2, 6), (3, 3), (4, 10)])
def test_against_setwise_model_on_tiny_inputs(oracle_mod, seed, R):
    n, S = 30, 3
    X = small_u8(n, 2, 100 + seed, 0, 12)                       # dense ties
    D = sqdist_matrix(X)
    snap = oracle_mod.random_graph(X, S, seed, R)
    model = lists_of(snap, n)
    for step in ["u", "u", "u", "r", "u", "u", "r", "u", "u", "u"]:
        if step == "u":
            snap, evals, _ = oracle_mod.update_neighbors_sync(X, snap, R)
            model, mevals = py_sync_round(D, model, R)
            assert evals == mevals
        else:
            snap = oracle_mod.add_reverse_edges(snap, R)
            model = py_add_reverse(D, model, R)
        assert lists_of(snap, n) == model


# ----------------------------------------------------------- search tooling
# ------------------------------- block-sequential passes (order of Alg. 4's vertex loop)
def test_vertex_order_worked_example(oracle_mod):
    g = read_golden("vertex_order_example.txt")
    X = np.array(g["points"], np.uint8)
    n = len(X)
    lists = [list(r) for r in g["initial_lists"]] + [[] for _ in range(n - len(g["initial_lists"]))]
    s0 = snapshot_from_lists(oracle_mod, X, lists, 8)

    def rows(s):
        got = [[i for _, i, _ in rows_of(s, u)] for u in range(n)]
        while got and not got[-1]:
            got.pop()
        return got

    s_in_place, ev, _ = oracle_mod.update_neighbors_blocks(X, s0, 8, n)
    assert rows(s_in_place) == g["in_place_rows_after"] and ev == g["in_place_evaluations"][0][0]
    assert rows_of(s_in_place, 2) == [(13.0, 3, 0)]             # received before its own turn: scanned, old
    assert rows_of(s_in_place, 1) == [(2.0, 2, 0)]
    s_sync, ev, _ = oracle_mod.update_neighbors_blocks(X, s0, 8, 1)
    assert rows(s_sync) == g["synchronous_rows_after"] and ev == g["synchronous_evaluations"][0][0]
    assert rows_of(s_sync, 1) == [(2.0, 2, 1), (13.0, 3, 0)]    # received after its scan: still new
    s_ref, ev_ref, _ = oracle_mod.update_neighbors_sync(X, s0, 8)
    assert rows(s_ref) == g["synchronous_rows_after"] and ev_ref == ev


def py_block_pass(D, lists, R, nblocks):
    """The pass in runs of consecutive ids, written with dicts: a run is scanned on the lists as they
    stand when it starts; its redirected edges are merged (existing entry wins, cut to R) before the next."""
    n = len(lists)
    bs = -(-n // nblocks)
    lists = [dict(l) for l in lists]
    evals = 0
    for lo in range(0, n, bs):
        incoming = {}
        kept = {}
        for u in range(lo, min(n, lo + bs)):
            sel = []
            for v in sorted(lists[u], key=lambda v: (D[u, v], v)):
                ok = True
                for w in sel:
                    if lists[u][v] == 0 and lists[u][w] == 0:
                        continue
                    evals += 1
                    if D[u, v] >= D[v, w]:
                        incoming.setdefault(w, set()).add(v)
                        ok = False
                        break
                if ok:
                    sel.append(v)
            kept[u] = {v: 0 for v in sel}
        for u, k in kept.items():
            lists[u] = k
        for x, vs in incoming.items():
            cand = {v: 1 for v in vs}
            cand.update(lists[x])
            order = sorted(cand, key=lambda v: (D[x, v], v))[:R]
            lists[x] = {v: cand[v] for v in order}
    return lists, evals


@pytest.mark.parametrize("seed,R,nblocks", [(1, 4, 1), (2, 6, 3), (3, 3, 7), (4, 10, 30), (5, 5, 4), (6, 8, 29)])
def test_block_passes_against_setwise_model(oracle_mod, seed, R, nblocks):
    n, S = 30, 3
    X = small_u8(n, 2, 200 + seed, 0, 12)                       # dense ties
    D = sqdist_matrix(X)
    snap = oracle_mod.random_graph(X, S, seed, R)
    model = lists_of(snap, n)
    for step in ["u", "u", "u", "r", "u", "u", "r", "u", "u"]:
        if step == "u":
            snap, evals, _ = oracle_mod.update_neighbors_blocks(X, snap, R, nblocks)
            model, mevals = py_block_pass(D, model, R, nblocks)
            assert evals == mevals
        else:
            snap = oracle_mod.add_reverse_edges(snap, R)
            model = py_add_reverse(D, model, R)
        assert lists_of(snap, n) == model


@pytest.mark.parametrize("kind", ["u8", "f32"])
def test_one_block_is_the_synchronous_round_and_n_blocks_the_in_place_order(oracle_mod, kind):
    n, S, T1, T2 = 150, 6, 3, 4
    X = small_u8(n, 8, 31, 0, 40) if kind == "u8" else small_f32(n, 8, 32)
    R = 40
    a = oracle_mod.build_blocks(X, S, R, T1, T2, 9, 1)
    b = oracle_mod.build_sync(X, S, R, T1, T2, 9)
    assert (a.snap.ids == b.snap.ids).all() and (a.snap.dist == b.snap.dist).all()
    assert (a.snap.flags == b.snap.flags).all() and (a.snap.deg == b.snap.deg).all()
    assert (a.round_evals == b.round_evals).all() and (a.round_props == b.round_props).all()
    # with lists that never reach the cut (R = n - 1) the n-block form is Alg. 4 as printed
    R = n - 1
    c = oracle_mod.build_blocks(X, S, R, T1, T2, 9, n)
    ids, deg, evals, mx = oracle_mod.build_paper_order(X, S, R, T1, T2, 9, R)
    assert mx <= R
    assert (c.snap.deg == deg).all() and (c.snap.ids == ids).all()
    assert int(c.round_evals.sum()) == evals
    # and the order matters: the two ends differ on the same input
    d = oracle_mod.build_blocks(X, S, R, T1, T2, 9, 1)
    assert (d.snap.ids != c.snap.ids).any()


@pytest.mark.parametrize("seed,R,M", [(1, 4, 4), (2, 4, 9), (3, 3, 29), (4, 6, 7), (5, 2, 9)])
def test_wide_merges_against_setwise_model(oracle_mod, seed, R, M):
    """Merges that cut to M >= R while Alg. 5 cuts to R: the whole build against the dict-based models of
    one round (cap M) and of AddReverseEdges (cap R); M = R is the synchronous build."""
    n, S, T1, T2 = 30, min(3, R), 3, 3
    X = small_u8(n, 2, 300 + seed, 0, 12)
    D = sqdist_matrix(X)
    got = oracle_mod.build_wide(X, S, R, M, T1, T2, seed)
    model = lists_of(oracle_mod.random_graph(X, S, seed, M), n)
    evals = []
    for t1 in range(T1):
        for _ in range(T2):
            model, ev = py_sync_round(D, model, M)
            evals.append(ev)
        if t1 != T1 - 1:
            model = py_add_reverse(D, model, R)
    assert lists_of(got.snap, n) == model and got.round_evals.tolist() == evals
    if M == R:
        ref = oracle_mod.build_sync(X, S, R, T1, T2, seed)
        assert (ref.snap.ids == got.snap.ids).all() and (ref.snap.deg == got.snap.deg).all()
    if (R, M) == (2, 9):
        # where lists do outgrow R between two AddReverseEdges calls, the wider merges change the graph
        ref = oracle_mod.build_sync(X, S, R, T1, T2, seed)
        assert (ref.snap.ids != got.snap.ids[:, :R]).any() or (ref.snap.deg != got.snap.deg).any()


def test_bruteforce_knn_matches_numpy(oracle_mod):
    X = small_u8(500, 16, 41)
    Q = small_u8(20, 16, 42)
    got = oracle_mod.bruteforce_knn(X, Q, 10)
    D = ((Q.astype(np.int64)[:, None, :] - X.astype(np.int64)[None, :, :]) ** 2).sum(-1)
    for q in range(len(Q)):
        want = sorted(range(len(X)), key=lambda i: (D[q, i], i))[:10]
        assert got[q].tolist() == want


def test_search_with_full_candidate_list_is_exact(oracle_mod):
    X = small_f32(200, 8, 51)
    Q = small_f32(10, 8, 52)
    res = oracle_mod.build_sync(X, 5, 12, 2, 3, 1)
    found, _ = oracle_mod.search(X, res.snap.ids, res.snap.deg, Q, 200, 12, 10)
    assert (found == oracle_mod.bruteforce_knn(X, Q, 10)).all()


def _search_model(X, ids, deg, q, start, L, K, k):
    """Alg. 1 with the cap of Eq. 4, written on Python sets and dicts (a different shape from the C
    routine: no sorted array, no insertion): C maps vertex -> distance, `visited` are the expanded members
    of C, `evaluated` every vertex whose distance to q was ever computed."""
    Xl = X.astype(np.int64)
    dist = lambda v: int(((Xl[v] - q.astype(np.int64)) ** 2).sum())
    C = {int(v): dist(int(v)) for v in start}
    evaluated, visited = set(C), set()
    evals = len(C)
    while True:
        pending = [v for v in C if v not in visited]
        if not pending:
            break
        u = min(pending, key=lambda v: (C[v], v))                        # select
        visited.add(u)
        for v in ids[u][:min(int(deg[u]), K)].tolist():                  # expand, with Eq. 4
            if v in evaluated:                                           # evaluated before
                continue
            evaluated.add(v)
            C[v] = dist(v)                                               # evaluate
            evals += 1
            if len(C) > L:                                               # C keeps its L nearest
                worst = max(C, key=lambda w: (C[w], w))
                del C[worst]
                visited.discard(worst)
    best = sorted(C, key=lambda v: (C[v], v))[:k]
    return best + [-1] * (k - len(best)), evals


@pytest.mark.parametrize("L,K,k", [(8, 4, 5), (16, 100, 10), (40, 6, 10), (5, 3, 5)])
def test_search_matches_a_setwise_model_on_small_inputs(oracle_mod, L, K, k):
    """The search routine against an independent model of Alg. 1 + Eq. 4 (only the seeded start set, which
    the paper leaves open, is taken from the generator that has its own pins)."""
    X = small_u8(300, 12, 61)
    Q = small_u8(15, 12, 62)
    g = oracle_mod.build_sync(X, 6, 16, 2, 3, 9).snap
    seed = 77
    found, evals = oracle_mod.search(X, g.ids, g.deg, Q, L, K, k, seed)
    total = 0
    for qi in range(len(Q)):
        start = oracle_mod.random_ids(len(X) + 1, len(X), min(L, len(X)), (seed + 0x9E3779B97F4A7C15 * qi) % 2 ** 64)
        want, ev = _search_model(X, g.ids, g.deg, Q[qi], start, L, K, k)
        assert found[qi].tolist() == want, "query %d" % qi
        total += ev
    assert evals == total


@pytest.mark.parametrize("name,n,nq", [("cfg1", 5000, 100), ("cfg2", 20000, 200)])
def test_search_quality_sync_vs_paper_order_vs_no_reverse_edges(oracle_mod, name, n, nq):
    """cfg1 as it is, and cfg2's generator and parameters (S=20 R=96 T1=4 T2=15) on its first 20,000 rows."""
    c = wl.CONFIGS[name]
    X, Q = wl.make_data(c, n), wl.make_queries(c, nq)
    gt = oracle_mod.bruteforce_knn(X, Q, 10)

    def recall(ids, deg, L=64):
        f, _ = oracle_mod.search(X, ids, deg, Q, L, 32, 10)
        return oracle_mod.recall_at_k(f, gt)

    sync = oracle_mod.build_sync(X, c.S, c.R, c.T1, c.T2, wl.BUILD_SEED).snap
    pids, pdeg, _, _ = oracle_mod.build_paper_order(X, c.S, c.R, c.T1, c.T2, wl.BUILD_SEED, 256)
    init = oracle_mod.random_graph(X, c.S, wl.BUILD_SEED, c.R)
    t1only = oracle_mod.build_sync(X, c.S, c.R, 1, c.T1 * c.T2, wl.BUILD_SEED).snap
    r_sync, r_paper = recall(sync.ids, sync.deg), recall(pids, pdeg)
    r_init, r_t1 = recall(init.ids, init.deg), recall(t1only.ids, t1only.deg)
    print("%s: recall@10 sync %.4f, paper order %.4f, T1 = 1 %.4f, random init %.4f" % (name, r_sync, r_paper, r_t1, r_init))
    assert r_sync > 0.97 and r_paper > 0.97
    assert abs(r_sync - r_paper) < 0.03                          # same method, different update order
    assert r_init < 0.5 < r_sync
    assert r_t1 <= r_sync                                        # Sec. 5.4: T1 = 1 is the worst setting
