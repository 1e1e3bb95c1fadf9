"""Scale check (Sec. 5.5 of the paper: a 20M-point dataset): N = 20,000,000 x 128 uint8 from cfg3's generator, the
paper's S, R, T1, T2, in the launch configuration the benchmark times.  A full oracle build would take about
an hour, so the GPU is driven through the build step by step and sampled:
  * UpdateNeighbors rounds: a closed sample (sampled targets + every vertex that lists one) is cut out of the
    device snapshot, relabelled to a compact problem (the map keeps the order of the ids, so every (delta, id)
    comparison, tie and cut is unchanged), run through the oracle, and the targets' complete new rows are
    compared key for key;
  * AddReverseEdges: for sampled vertices the union with the reversed edges and the cut to R are written out in
    numpy from the device's pre-state; the GPU's row must be that list minus only edges whose target ended up
    with exactly R incoming edges (where the in-degree cut of Alg. 5 acted); out- and in-degrees <= R everywhere.
"""
import numpy as np
import pytest

import workloads as wl
from conftest import live
from gpu_util import dist_bits_of

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rn():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2310_20419_amd as m
    m.load_library()
    return m


def _ids_of(keys, deg):
    """Neighbour ids of a device snapshot as int32, 0 in the unused slots, and the mask of the used ones."""
    import torch
    valid = torch.arange(keys.shape[1], device=keys.device)[None, :] < deg[:, None]
    ids = ((keys >> 1) & 0x7FFFFFFF).to(torch.int32)
    ids.masked_fill_(~valid, 0)
    return ids, valid


def _points_into(ids, valid, members, n):
    """Mask of the used slots whose id is one of `members` (a table lookup: no sort of the whole graph)."""
    import torch
    mark = torch.zeros(n, dtype=torch.bool, device=ids.device)
    mark[members.to(torch.int64)] = True
    return mark[ids] & valid


def compact_round_check(rn, oracle_mod, X, Xd, keys, deg, R, targets, is_float, what):
    """One UpdateNeighbors round on the GPU, checked on a closed sample through a compact oracle problem."""
    import torch
    dev = keys.device
    tt = torch.from_numpy(targets.astype(np.int32)).to(dev)
    ids_dev, valid = _ids_of(keys, deg)
    sources = torch.nonzero(_points_into(ids_dev, valid, tt, keys.shape[0]).any(1)).flatten()
    del ids_dev, valid
    scanned = torch.unique(torch.cat([tt.to(torch.int64), sources]))              # ascending
    sub_deg = deg[scanned].cpu().numpy()
    ids_s, bits_s, flags_s = rn.unpack_keys(keys[scanned].cpu().numpy().view(np.uint64), sub_deg)
    scanned = scanned.cpu().numpy()
    ref = np.unique(np.concatenate([ids_s[ids_s >= 0].astype(np.int64), scanned]))  # ascending: a monotone relabelling
    snap = oracle_mod.Snapshot.empty(len(ref), R)
    rows = np.searchsorted(ref, scanned)
    snap.ids[rows] = np.where(ids_s >= 0, np.searchsorted(ref, np.maximum(ids_s, 0)), -1)
    snap.dist[rows] = bits_s.view(np.float32).astype(np.float64) if is_float else bits_s.astype(np.float64)
    snap.flags[rows] = flags_s
    snap.deg[rows] = sub_deg
    want, _, _ = oracle_mod.update_neighbors_sync(np.ascontiguousarray(X[ref]), snap, R)
    rn.rnnd_update_neighbors(Xd, keys, deg, R, 1)
    tdeg = deg[tt.to(torch.int64)].cpu().numpy()
    ids_a, bits_a, flags_a = rn.unpack_keys(keys[tt.to(torch.int64)].cpu().numpy().view(np.uint64), tdeg)
    trow = np.searchsorted(ref, targets)
    want_bits = dist_bits_of(want.dist, is_float)
    for i, t in enumerate(targets):
        m = want.deg[trow[i]]
        assert tdeg[i] == m, "%s: vertex %d has %d entries, the oracle %d" % (what, t, tdeg[i], m)
        assert (ids_a[i, :m] == ref[want.ids[trow[i], :m]]).all(), "%s: ids of vertex %d" % (what, t)
        assert (bits_a[i, :m] == want_bits[trow[i], :m]).all(), "%s: distances of vertex %d" % (what, t)
        assert (flags_a[i, :m] == want.flags[trow[i], :m]).all(), "%s: flags of vertex %d" % (what, t)
    print("%s: %d complete rows identical to the oracle's (closed sample of %d lists over %d vertices)"
          % (what, len(targets), len(scanned), len(ref)), flush=True)


def reverse_union_check(rn, keys, deg, R, sample, what):
    """AddReverseEdges on the GPU; the sampled rows against the union and cut written out in numpy."""
    import torch
    dev = keys.device
    n = keys.shape[0]
    st = torch.from_numpy(sample.astype(np.int32)).to(dev)
    ids_dev, valid = _ids_of(keys, deg)
    hit = torch.nonzero(_points_into(ids_dev, valid, st, n))                   # (u, slot) of every edge into the sample
    src = hit[:, 0].cpu().numpy()
    tgt = ids_dev[hit[:, 0], hit[:, 1]].cpu().numpy()
    ekey = keys[hit[:, 0], hit[:, 1]].cpu().numpy().view(np.uint64)
    del ids_dev, valid, hit
    sdeg = deg[st.to(torch.int64)].cpu().numpy()
    srows = keys[st.to(torch.int64)].cpu().numpy().view(np.uint64)
    expect = {}
    for i, x in enumerate(sample):
        own = srows[i, :sdeg[i]]
        sel = tgt == x
        rev = ((ekey[sel] >> np.uint64(32)) << np.uint64(32)) | (src[sel].astype(np.uint64) << np.uint64(1)) | np.uint64(1)
        allk = np.sort(np.concatenate([own, rev]))                            # old before new for the same (delta, id)
        keep = np.ones(len(allk), bool)
        keep[1:] = (allk[1:] >> np.uint64(1)) != (allk[:-1] >> np.uint64(1))  # an existing entry wins
        expect[int(x)] = allk[keep][:R]
    rn.rnnd_add_reverse_edges(keys, deg, R)
    ids_dev, valid = _ids_of(keys, deg)
    indeg = torch.bincount(ids_dev[valid].to(torch.int64), minlength=n)
    assert int(deg.max()) <= R and int(indeg.max()) <= R                      # Alg. 5; Sec. 5.3
    del ids_dev, valid
    pdeg = deg[st.to(torch.int64)].cpu().numpy()
    prows = keys[st.to(torch.int64)].cpu().numpy().view(np.uint64)
    indeg_h = indeg.cpu().numpy()
    cut = 0
    for i, x in enumerate(sample):
        got, exp = prows[i, :pdeg[i]], expect[int(x)]
        missing = np.setdiff1d(exp, got)
        assert np.isin(got, exp).all() and (np.diff(got.astype(np.int64)) != 0).all(), "%s: vertex %d" % (what, x)
        assert (got == exp[np.isin(exp, got)]).all(), "%s: order of vertex %d" % (what, x)
        for k in missing:           # dropped by the in-degree cut: its target is full
            v = int((int(k) >> 1) & 0x7FFFFFFF)
            assert indeg_h[v] == R, "%s: vertex %d lost its edge to %d, which has %d incoming edges" % (what, x, v, indeg_h[v])
        cut += len(missing)
    print("%s: %d sampled rows = union with reversed edges cut to R (%d edges removed by the in-degree cut); "
          "max out-degree %d, max in-degree %d" % (what, len(sample), cut, int(deg.max()), int(indeg.max())), flush=True)


def test_the_sampling_checks_on_a_graph_the_oracle_can_build_whole(rn, oracle_mod):
    """The two sampled checks at a size where the whole graph is also compared with the oracle: 30,000 rows."""
    _stepwise_sampled(rn, oracle_mod, 30_000, 2, 3, 60, 120, full=True)


@pytest.mark.slow
@live
def test_20m_rows_sampled_parity(rn, oracle_mod):
    _stepwise_sampled(rn, oracle_mod, 20_000_000, wl.CONFIGS["cfg3"].T1, wl.CONFIGS["cfg3"].T2, 300, 500, full=False)


def _stepwise_sampled(rn, oracle_mod, n, T1, T2, n_targets, n_reverse, full):
    import dataclasses
    import time
    import torch
    from gpu_util import assert_snapshot_equal
    c = dataclasses.replace(wl.CONFIGS["cfg3"], N=n, T1=T1, T2=T2)
    t0 = time.time()
    X = wl.make_data(c)
    print("%d x 128 uint8 generated in %.0f s" % (n, time.time() - t0), flush=True)
    Xd = torch.from_numpy(X).cuda()
    R, T1, T2 = c.R, c.T1, c.T2
    g = np.random.default_rng(20)
    keys, deg = rn.rnnd_random_graph(Xd, c.S, R, wl.BUILD_SEED)
    sample = np.sort(g.choice(n, min(300, n), replace=False))
    rows0 = keys[torch.from_numpy(sample).cuda()].cpu().numpy().view(np.uint64)
    for i, u in enumerate(sample):
        want_ids = oracle_mod.random_ids(n, int(u), c.S, wl.BUILD_SEED)
        assert sorted(((rows0[i, :c.S] >> np.uint64(1)) & np.uint64(0x7FFFFFFF)).tolist()) == sorted(want_ids.tolist())
    done = 0
    check_before = {0, min(3, T2 - 1), T2, T1 * T2 - 1}
    for t1 in range(T1):
        for t2 in range(T2):
            if done in check_before:
                targets = np.sort(g.choice(n, n_targets, replace=False))
                compact_round_check(rn, oracle_mod, X, Xd, keys, deg, R, targets, False, "N %d round %d" % (n, done + 1))
            else:
                rn.rnnd_update_neighbors(Xd, keys, deg, R, 1)
            done += 1
        if t1 != T1 - 1:
            if t1 == 0:
                reverse_union_check(rn, keys, deg, R, np.sort(g.choice(n, n_reverse, replace=False)),
                                    "N %d AddReverseEdges 1" % n)
            else:
                rn.rnnd_add_reverse_edges(keys, deg, R)
    graph, degree, fkeys, st = rn.rnnd_build_ex(Xd, c.S, R, T1, T2, wl.BUILD_SEED)
    print("gpu build done: %.1f ms, mean degree %.2f" % (st.total_ms, float(degree.float().mean())), flush=True)
    pad = torch.arange(R, device="cuda")[None, :] >= degree[:, None]
    assert (degree == deg).all() and bool(((fkeys == keys) | pad).all())          # the step-wise path is the build's path
    if full:
        want = oracle_mod.build_sync(X, c.S, R, T1, T2, wl.BUILD_SEED)
        assert_snapshot_equal(want.snap, False, fkeys, degree, "whole graph at N = %d" % n)
