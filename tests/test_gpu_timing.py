"""Where the per-round times of the statistics come from: the device's own clock (the default, free) or HIP
events attached to the launches (rnnd_set_event_timing).  Both describe the same build."""
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


@pytest.mark.parametrize("kind,n,d", [("heavy_u8", 60000, 128), ("unit_f32", 30000, 96), ("heavy_u8", 20000, 48)])
def test_device_clock_and_event_times_describe_the_same_build(rn, kind, n, d):
    """Same graph and counters in both modes; every round has a scan time inside its round time; the rounds, the
    reverse calls and the initialisation together fit in the call's total; and the two clocks agree on the sum of
    the scan times (the device clock sees a scan end where the next kernel starts, so it may read a little more)."""
    import torch
    X = torch.from_numpy(wl.custom(kind, n, d, 11)).cuda()
    S, R, T1, T2 = 12, 48, 3, 5
    out = {}
    try:
        for mode in (False, True, False):
            rn.rnnd_set_event_timing(mode)
            rn.rnnd_build(X, S, R, T1, T2, 5)        # warm: the workspace block exists
            g, dg, _, st = rn.rnnd_build_ex(X, S, R, T1, T2, 5, want_keys=False)
            out[mode] = (g, dg, st.as_dict())
    finally:
        rn.rnnd_set_event_timing(False)
    (g0, d0, s0), (g1, d1, s1) = out[False], out[True]
    assert torch.equal(g0, g1) and torch.equal(d0, d1)
    # (not "dropped": a hub whose surplus streams through the merge may count an edge twice, depending on arrival order)
    for key in ("active", "proposals", "algo_evals", "exec_evals", "gathered_rows"):
        assert s0[key][:T1 * T2] == s1[key][:T1 * T2], key
    for s in (s0, s1):
        rounds = s["rounds"]
        assert rounds == T1 * T2
        for t in range(rounds):
            assert 0.0 < s["scan_ms"][t] <= s["round_ms"][t] * 1.001, (t, s["scan_ms"][t], s["round_ms"][t])
        for r in range(T1 - 1):
            assert s["reverse_ms"][r] > 0.0
        parts = sum(s["round_ms"][:rounds]) + sum(s["reverse_ms"][:T1 - 1]) + s["init_ms"]
        assert parts <= s["total_ms"] * 1.02 + 0.05, (parts, s["total_ms"])
        assert parts >= s["total_ms"] * 0.75, (parts, s["total_ms"])
    a, b = sum(s0["scan_ms"][:T1 * T2]), sum(s1["scan_ms"][:T1 * T2])
    print("scan time by device clock %.3f ms, by HIP events %.3f ms; total %.3f / %.3f ms"
          % (a, b, s0["total_ms"], s1["total_ms"]))
    assert b * 0.9 <= a <= b * 1.25 + 0.1, (a, b)


def test_statistics_cost_nothing_with_the_device_clock(rn):
    """The reason for the device clock: a build with statistics must not be slower than one without (events on
    every round's launches cost a few percent at this size; allow for timer noise only)."""
    import time
    import torch
    cfg = wl.CONFIGS["cfg2"]
    X = torch.from_numpy(wl.make_data(cfg)).cuda()

    def timed(fn, reps=8):
        fn()
        torch.cuda.synchronize()
        best = 1e9
        for _ in range(3):
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            best = min(best, (time.perf_counter() - t0) / reps)
        return best

    rn.rnnd_set_event_timing(False)
    plain = timed(lambda: rn.rnnd_build(X, cfg.S, cfg.R, cfg.T1, cfg.T2, wl.BUILD_SEED))
    with_stats = timed(lambda: rn.rnnd_build_ex(X, cfg.S, cfg.R, cfg.T1, cfg.T2, wl.BUILD_SEED, want_keys=False))
    print("cfg2 build: %.3f ms without statistics, %.3f ms with" % (plain * 1e3, with_stats * 1e3))
    assert with_stats <= plain * 1.04 + 2e-4, (plain, with_stats)


def test_step_wise_rounds_report_their_times(rn):
    """rnnd_update_neighbors fills round_ms and scan_ms of the rounds it ran (device clock)."""
    import torch
    X = torch.from_numpy(wl.custom("heavy_u8", 50000, 128, 5)).cuda()
    R, S, rounds = 48, 12, 4
    keys, deg = rn.rnnd_random_graph(X, S, R, 3)
    st = rn.rnnd_update_neighbors(X, keys, deg, R, rounds).as_dict()
    assert st["rounds"] == rounds
    for t in range(rounds):
        assert 0.0 < st["scan_ms"][t] <= st["round_ms"][t] * 1.001, (t, st["scan_ms"][t], st["round_ms"][t])
        assert st["round_ms"][t] < 50.0
    assert len(st["scan_ms"]) == rounds
