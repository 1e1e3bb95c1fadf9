"""The uint8 matrix-core scan of a round as several launches (short lists; one per longer class), as one launch
whose blocks are divided among all classes, or as the short-list launch plus one launch shared by the longer
classes.  The default picks by size, so the small parity tests exercise the second, the 1M tests the third and the 20M test
the first;
here each is forced on the same inputs and must give the oracle's graph, the oracle's evaluation and redirect
counts, and the same result as the others."""
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


def clustered_u8(n, d, seed, k=3, spread=9):
    g = np.random.default_rng(seed)
    c = g.integers(20, 236, size=(k, d))
    x = c[g.integers(0, k, size=n)] + g.integers(-spread, spread + 1, size=(n, d))
    return np.clip(x, 0, 255).astype(np.uint8)


CASES = [
    # data, S, R, T1, T2: R picks the number of long-list classes (<= 64: one, <= 96: two, <= 128: three)
    (lambda: wl.custom("heavy_u8", 3000, 128, 7), 20, 96, 3, 4),
    (lambda: clustered_u8(900, 64, 12), 40, 128, 3, 4),          # tight clusters: lists of every length up to 128
    (lambda: clustered_u8(1200, 32, 5), 30, 64, 2, 5),
    (lambda: wl.custom("heavy_u8", 2500, 128, 3), 50, 50, 2, 3),
    (lambda: wl.make_data(wl.CONFIGS["cfg1"]), 10, 32, 2, 4),    # R = 32: short lists only, the switch changes nothing
]


@pytest.mark.parametrize("case", range(len(CASES)))
def test_both_forms_give_the_oracles_build(rn, oracle_mod, case):
    make, S, R, T1, T2 = CASES[case]
    X = make()
    want = oracle_mod.build_sync(X, S, R, T1, T2, wl.BUILD_SEED)
    out = {}
    try:
        for mode in (1, 2, 3):
            rn.rnnd_set_scan_launches(mode)
            graph, degree, keys, st = rn.rnnd_build_ex(cuda(X), S, R, T1, T2, wl.BUILD_SEED)
            assert st.kernel_variant == 2
            assert_snapshot_equal(want.snap, False, keys, degree, "case %d mode %d" % (case, mode))
            assert list(st.algo_evals[:T1 * T2]) == want.round_evals.tolist()
            assert list(st.proposals[:T1 * T2]) == want.round_props.tolist()
            out[mode] = (graph, degree, st.as_dict())
    finally:
        rn.rnnd_set_scan_launches(0)
    import torch
    for mode in (2, 3):
        assert torch.equal(out[1][0], out[mode][0]) and torch.equal(out[1][1], out[mode][1])
        for key in ("active", "proposals", "algo_evals", "exec_evals", "gathered_rows"):
            assert out[1][2][key] == out[mode][2][key], (mode, key)


@pytest.mark.parametrize("n", [40_000, 600_000])
def test_both_forms_agree_at_sizes_on_either_side_of_the_default_rule(rn, n):
    """cfg2's generator at a size the default gives one launch and at a size it gives two: same graph, same
    counters whichever form is forced (the oracle check at such sizes is test_gpu_parity's)."""
    import torch
    cfg = wl.CONFIGS["cfg2"]
    X = cuda(wl.custom("heavy_u8", n, 128, 31))
    out = {}
    try:
        for mode in (0, 1, 2, 3):
            rn.rnnd_set_scan_launches(mode)
            g, dg, _, st = rn.rnnd_build_ex(X, cfg.S, cfg.R, 2, 6, wl.BUILD_SEED, want_keys=False)
            out[mode] = (g, dg, st.as_dict())
    finally:
        rn.rnnd_set_scan_launches(0)
    for mode in (1, 2, 3):
        assert torch.equal(out[0][0], out[mode][0]) and torch.equal(out[0][1], out[mode][1])
        for key in ("active", "proposals", "algo_evals", "exec_evals", "gathered_rows"):
            assert out[0][2][key] == out[mode][2][key], (mode, key)
