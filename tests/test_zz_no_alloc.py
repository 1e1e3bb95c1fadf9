"""rnnd_build_static: the build for callers that cannot allocate device memory.  Its workspace is a static
device array; the graph must be the one rnnd_build gives, bit for bit, on two calls in a row that share the
array (the second on a smaller input, so that it runs on what the first left behind)."""
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


def test_static_build_equals_the_allocating_build_twice_in_a_row(rn, oracle_mod):
    import torch
    c = wl.CONFIGS["cfg1"]
    X = wl.make_data(c)
    cases = [(X, c.S, c.R, c.T1, c.T2),                                   # 5,000 x 32 uint8, R = 32
             (X[:1800].copy(), 6, 16, 2, 3),                              # smaller, right after: same array
             (wl.custom("unit_f32", 1500, 96, 2), 8, 24, 2, 3),           # float rows
             (wl.custom("heavy_u8", 9000, 128, 8), 20, 96, 2, 4)]         # paper's R; close to the limit
    for Xh, S, R, T1, T2 in cases:
        Xd = torch.from_numpy(Xh).cuda()
        n = len(Xh)
        need = rn.rnnd_workspace_bytes(n, Xh.shape[1], rn.RNND_U8 if Xh.dtype == np.uint8 else rn.RNND_F32, R, T1 * T2)
        assert need <= rn.RNND_STATIC_SCRATCH_BYTES
        graph = torch.full((n, R), -7, dtype=torch.int32, device="cuda")
        degree = torch.full((n,), -7, dtype=torch.int32, device="cuda")
        # no device allocation during the call: the library's kept workspace block is released first (so that
        # the call cannot be served from it), and the device's free memory must not drop across the call
        import gc
        gc.collect()
        rn.rnnd_release_workspace()
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        rn.rnnd_build_static(Xd, S, R, T1, T2, wl.BUILD_SEED, graph, degree)
        assert torch.cuda.mem_get_info()[0] >= free_before
        g0, d0 = rn.rnnd_build(Xd, S, R, T1, T2, wl.BUILD_SEED)
        assert (graph == g0).all() and (degree == d0).all(), (n, R)
        want = oracle_mod.build_sync(Xh, S, R, T1, T2, wl.BUILD_SEED)
        assert (graph.cpu().numpy() == want.snap.ids).all() and (degree.cpu().numpy() == want.snap.deg).all()


def test_static_build_rejects_what_does_not_fit(rn):
    import torch
    X = torch.zeros((40_000, 128), dtype=torch.uint8, device="cuda")
    assert rn.rnnd_workspace_bytes(40_000, 128, rn.RNND_U8, 96, 60) > rn.RNND_STATIC_SCRATCH_BYTES
    graph = torch.empty((40_000, 96), dtype=torch.int32, device="cuda")
    degree = torch.empty((40_000,), dtype=torch.int32, device="cuda")
    with pytest.raises(rn.RnndError) as e:
        rn.rnnd_build_static(X, 20, 96, 4, 15, 1, graph, degree)
    assert e.value.status == -7 and "scratch" in str(e.value)
