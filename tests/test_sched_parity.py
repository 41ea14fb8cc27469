"""Library scheduler (C ABI of include/gpulet_sched.h) against the plain-Python
oracle, decision by decision: integers bit-exact, rates and cycles to 1e-12
relative (both sides are fp64 and take every comparison in fp64).  Host-only
code: no GPU needed."""

import ctypes

import pytest

from oracle import scheduling as S
from paper_2109_01611_amd import gpulet, inputs, scenarios, sched

SIZES, BATCHES = list(scenarios.SIZES), list(scenarios.BATCHES)


def random_problem(seed, n_models, n_gpu, with_intf, merge, load=1.5):
    tabs = [scenarios.synthetic_table(seed, "m%d" % i) for i in range(n_models)]
    slos = [scenarios.slo_from_table(t) for t in tabs]
    u = inputs.uniform(seed, "rates", n_models + n_models * n_models)
    rates = []
    for i in range(n_models):
        full = 1000.0 * 32 / tabs[i][-1][-1]
        rates.append(0.0 if u[i] < 0.15 else float(full * load * u[i]))
    F = None
    if with_intf:
        F = [[float(0.3 * u[n_models + a * n_models + b] ** 3) for b in range(n_models)] for a in range(n_models)]
    return tabs, rates, slos, n_gpu, F, merge


def both(tabs, rates, slos, n_gpu, F, merge):
    want = S.elastic_partitioning(S.Problem(SIZES, BATCHES, tabs, rates, slos, n_gpu, intf=F, merge=merge))
    got = sched.elastic_partitioning(SIZES, BATCHES, tabs, rates, slos, n_gpu, slowdown=F, merge=merge)
    return want, got


def assert_same(want, got):
    assert got[0] == want[0]
    assert len(got[1]) == len(want[1])
    for g, w in zip(got[1], want[1]):
        assert g[:5] == w[:5]
        assert g[5] == pytest.approx(w[5], rel=1e-12, abs=0.0)
        assert g[6] == pytest.approx(w[6], rel=1e-12, abs=0.0)


def test_curve_knee_and_required_size_match_on_synthetic_tables():
    for seed in range(200):
        tab = scenarios.synthetic_table(seed, "curve")
        slo = scenarios.slo_from_table(tab) * (0.3 + 0.01 * seed)
        want = S.rate_curve(tab, BATCHES, slo)
        got = sched.rate_curve(BATCHES, tab, slo)
        assert got == want                                   # same expression order: bit-exact
        for i, row in enumerate(tab):
            for f in (0.0, 0.07):
                r, j = S.affordable_rate(row, BATCHES, slo, f)
                assert sched.affordable_rate(BATCHES, row, slo, f) == (r, BATCHES[j] if j >= 0 else 0)
        p_eff, curv = sched.max_efficient_partition(SIZES, got, with_curvature=True)
        assert p_eff == S.max_efficient_partition(SIZES, want)
        assert curv == S.curvature(S.normalised([float(s) for s in SIZES]), S.normalised(want))
        for frac in (0.0, 0.1, 0.5, 0.9, 1.0, 1.5):
            w = frac * max(want)
            assert sched.min_required_partition(SIZES, got, w) == S.min_required_partition(SIZES, want, w)


def test_knee_special_cases_match():
    for rates in ([3.0 * s for s in SIZES], [float(s * s) for s in SIZES], [5.0] * 6, [0.0] * 6,
                  [100.0, 200.0, 250.0, 260.0, 270.0, 280.0]):
        assert sched.max_efficient_partition(SIZES, rates) == S.max_efficient_partition(SIZES, rates)
    assert sched.max_efficient_partition([20, 40, 60, 80, 100], [0.0, 3.0, 4.0, 7.0, 8.0]) == 40
    assert sched.max_efficient_partition([50, 100], [1.0, 2.0]) == 100
    assert sched.max_efficient_partition([100], [1.0]) == 100


@pytest.mark.parametrize("with_intf", [False, True])
@pytest.mark.parametrize("merge", [False, True])
def test_elastic_partitioning_matches_the_oracle_on_random_scenarios(with_intf, merge):
    outcomes = set()
    merged = 0
    for seed in range(400):
        args = random_problem(seed, 1 + seed % 5, 1 + (seed // 5) % 4, with_intf, merge,
                              load=(0.05, 0.4, 1.5)[seed % 3])
        want, got = both(*args)
        assert_same(want, got)
        outcomes.add(want[0])
        merged += any(e[6] > 0 for e in want[1])
    assert outcomes == {True, False}
    assert (merged > 20) if merge else (merged == 0)


def test_whole_gpus_only_matches_the_oracle():
    n_ok = 0
    for seed in range(150):
        tabs, rates, slos, n_gpu, F, merge = random_problem(seed, 2 + seed % 4, 1 + seed % 3, False, True, load=0.2)
        tabs = [[t[-1]] for t in tabs]
        want = S.elastic_partitioning(S.Problem([100], BATCHES, tabs, rates, slos, n_gpu, merge=True))
        got = sched.elastic_partitioning([100], BATCHES, tabs, rates, slos, n_gpu, merge=True)
        assert_same(want, got)
        n_ok += want[0]
    assert 10 < n_ok < 150


def test_hand_worked_cases_match():
    scal = lambda per: [[per * b * 100.0 / p for b in BATCHES] for p in SIZES]
    knee = lambda per, k: [[per * b * 100.0 / min(p, k) for b in BATCHES] for p in SIZES]
    ok, e = sched.elastic_partitioning(SIZES, BATCHES, [scal(1.0)], [150.0], [1000.0], 1)
    assert ok and e == [(0, 20, 0, 0, 32, 150.0, 0.0)]
    ok, e = sched.elastic_partitioning(SIZES, BATCHES, [knee(1.0, 40)], [900.0], [1000.0], 2)
    assert ok and [(x[0], x[1], x[2]) for x in e] == [(0, 40, 0), (0, 60, 1), (1, 20, 0)]
    ok, e = sched.elastic_partitioning(SIZES, BATCHES, [scal(0.1), scal(0.1)], [100.0, 100.0], [50.0, 50.0], 1)
    assert ok and [(x[0], x[1], x[2], x[3], x[4]) for x in e] == [(0, 20, 0, 0, 1), (0, 20, 0, 1, 1)]
    assert e[0][6] == e[1][6] == pytest.approx(1.0)
    assert sched.elastic_partitioning(SIZES, BATCHES, [scal(1.0)], [10.0], [1.9], 4) == (False, [])
    assert sched.elastic_partitioning(SIZES, BATCHES, [scal(1.0)], [0.0], [100.0], 1) == (True, [])


def test_paper_rate_grid_matches_on_a_five_model_set():
    tabs = [scenarios.synthetic_table(11, n) for n in scenarios.MODELS]
    slos = [scenarios.slo_from_table(t) for t in tabs]
    full = [1000.0 * 32 / t[-1][-1] for t in tabs]
    grid = scenarios.rate_grid(5, levels=(0.0, 1.0, 2.0, 3.0))
    assert len(grid) == 1023
    n_ok = 0
    for levels in grid[::7]:
        rates = [l * f * 0.3 for l, f in zip(levels, full)]
        want, got = both(tabs, rates, slos, 4, None, True)
        assert_same(want, got)
        n_ok += want[0]
    assert 0 < n_ok < len(grid[::7])


def test_argument_errors():
    tab = scenarios.synthetic_table(0, "e")
    with pytest.raises(gpulet.GpuletError):
        sched.affordable_rate([1, 1, 2], [1.0, 2.0, 3.0], 10.0)            # batches not ascending
    with pytest.raises(gpulet.GpuletError):
        sched.affordable_rate([1, 2], [1.0, -2.0], 10.0)                   # latency not positive
    with pytest.raises(gpulet.GpuletError):
        sched.affordable_rate([1, 2], [1.0, 2.0], 0.0)                     # SLO not positive
    with pytest.raises(gpulet.GpuletError):
        sched.max_efficient_partition([40, 20, 100], [1.0, 2.0, 3.0])
    with pytest.raises(gpulet.GpuletError):
        sched.elastic_partitioning([20, 50, 100], BATCHES, [[r[:] for r in tab[:3]]], [1.0], [10.0], 1)  # no 80
    with pytest.raises(gpulet.GpuletError):
        sched.elastic_partitioning(SIZES[:-1], BATCHES, [tab[:-1]], [1.0], [10.0], 1)   # does not end at 100
    with pytest.raises(gpulet.GpuletError):
        sched.elastic_partitioning(SIZES, BATCHES, [tab], [-1.0], [10.0], 1)
    with pytest.raises(gpulet.GpuletError):
        sched.elastic_partitioning(SIZES, BATCHES, [tab], [1.0], [10.0], 0)
    with pytest.raises(gpulet.GpuletError):
        sched.elastic_partitioning(SIZES, BATCHES, [tab], [1.0], [10.0], 1, slowdown=[[-0.1]])
    n, ok = ctypes.c_int(), ctypes.c_int()
    assert gpulet.lib.gpulet_elastic_partitioning(None, None, 0, ctypes.byref(n), ctypes.byref(ok)) == gpulet.EINVAL
    # too small an output array reports how many entries are needed
    full = 1000.0 * 32 / tab[-1][-1]
    with pytest.raises(gpulet.GpuletError) as ei:
        sched.elastic_partitioning(SIZES, BATCHES, [tab], [3.5 * full], [scenarios.slo_from_table(tab)], 8,
                                   max_entries=1)
    assert ei.value.status == gpulet.ENOMEM
