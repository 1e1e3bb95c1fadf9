"""The library's own device memory: the workspace block kept between calls, what a call may assume about its
contents (nothing), and what happens when it cannot be had."""
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


def cuda(a):
    import torch
    return torch.from_numpy(a).cuda()


@pytest.fixture
def poisoned(rn):
    """Every workspace is filled with 0xA5 bytes before the call clears what it needs cleared."""
    rn.rnnd_release_workspace()
    rn.rnnd_set_workspace_poison(True)
    yield
    rn.rnnd_set_workspace_poison(False)
    rn.rnnd_release_workspace()


@pytest.mark.parametrize("name", ["u8", "f32"])
def test_every_entry_point_clears_what_it_relies_on(rn, oracle_mod, poisoned, name):
    """Regression: AddReverseEdges takes arrival numbers from a per-vertex counter that must read zero; the
    step-wise entry point once left it as allocated.  With the workspace poisoned, every step-wise entry point
    and the builds must still give the oracle's result, each as the FIRST call on a fresh block and again on
    the block the previous call left behind."""
    X = wl.custom("heavy_u8", 2500, 128, 3) if name == "u8" else wl.custom("unit_f32", 2500, 96, 4)
    isf = X.dtype == np.float32
    R, S = 24, 10
    Xd = cuda(X)
    snap = oracle_mod.random_graph(X, S, 5, R)
    for first in ("r", "u", "b"):
        rn.rnnd_release_workspace()                   # the next call allocates (and poisons) a fresh block
        s = snap
        for step in (first, "r", "u", "b", "r", "u"):
            keys, deg = snapshot_to_device(s, isf, R)
            if step == "u":
                s, evals, props = oracle_mod.update_neighbors_sync(X, s, R)
                st = rn.rnnd_update_neighbors(Xd, keys, deg, R, 1)
                assert st.algo_evals[0] == evals and st.proposals[0] == props
            elif step == "b":
                s, evals, props = oracle_mod.update_neighbors_blocks(X, s, R, 3)
                st = rn.rnnd_update_neighbors_blocks(Xd, keys, deg, R, 3, 1)
                assert st.algo_evals[0] == evals and st.proposals[0] == props
            else:
                s = oracle_mod.add_reverse_edges(s, R)
                rn.rnnd_add_reverse_edges(keys, deg, R)
            assert_snapshot_equal(s, isf, keys, deg, "%s first %s step %s" % (name, first, step))
    want = oracle_mod.build_sync(X, S, R, 3, 3, 9)
    for _ in range(2):
        graph, degree, keys, st = rn.rnnd_build_ex(Xd, S, R, 3, 3, 9)
        assert_snapshot_equal(want.snap, isf, keys, degree, name + " build on a poisoned workspace")
    wantb = oracle_mod.build_blocks(X, S, R, 2, 3, 9, 4)
    graph, degree, keys, st = rn.rnnd_build_blocks(Xd, S, R, 2, 3, 9, 4)
    assert_snapshot_equal(wantb.snap, isf, keys, degree, name + " block-sequential build on a poisoned workspace")
    wantw = oracle_mod.build_wide(X, S, 12, R, 2, 3, 9)
    graph, degree, keys, st = rn.rnnd_build_wide(Xd, S, 12, R, 2, 3, 9)
    assert_snapshot_equal(wantw.snap, isf, keys, degree, name + " wide build on a poisoned workspace")


def test_the_kept_block_grows_shrinks_and_is_released(rn):
    """A small build after a large one, a large one after a small one, and a release in between all give the
    same graphs: the kept block carries nothing from call to call."""
    import torch
    c = wl.CONFIGS["cfg1"]
    X = cuda(wl.make_data(c))
    Xs = X[:700].contiguous()
    g_big, d_big = rn.rnnd_build(X, c.S, c.R, c.T1, c.T2, 3)
    g_small, d_small = rn.rnnd_build(Xs, c.S, c.R, c.T1, c.T2, 3)           # reuses the larger block
    rn.rnnd_release_workspace()
    g_small2, d_small2 = rn.rnnd_build(Xs, c.S, c.R, c.T1, c.T2, 3)         # allocates a small one
    g_big2, d_big2 = rn.rnnd_build(X, c.S, c.R, c.T1, c.T2, 3)              # replaces it by a larger one
    assert (g_small == g_small2).all() and (d_small == d_small2).all()
    assert (g_big == g_big2).all() and (d_big == d_big2).all()
    rn.rnnd_release_workspace()
    rn.rnnd_release_workspace()                                              # nothing kept: a no-op
    torch.cuda.synchronize()


def test_allocation_failure_is_reported_not_fatal(rn):
    """A workspace larger than the device's memory (about 400 GB here) is RNND_ERR_OOM from the allocator; the
    library stays usable afterwards."""
    import torch
    n = 600_000_000
    X = torch.zeros((n, 1), dtype=torch.uint8, device="cuda")
    assert rn.rnnd_workspace_bytes(n, 1, rn.RNND_U8, 3, 1) > 330 * 2**30
    with pytest.raises(rn.RnndError) as e:
        rn.rnnd_build(X, 1, 3, 1, 1, 0)
    assert e.value.status == -5
    del X
    c = wl.CONFIGS["cfg1"]
    Xs = cuda(wl.make_data(c))
    g, d = rn.rnnd_build(Xs, c.S, c.R, c.T1, c.T2, 3)
    assert int(d.min()) >= 1
