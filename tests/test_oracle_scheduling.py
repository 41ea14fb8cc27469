"""Pins of the scheduler oracle (paper Sec. 2.2, Sec. 4.3, Algorithm 1) against
things other than itself: closed forms, an event-by-event replay of batched
serving, hand-worked allocations and the invariants of a valid schedule."""

import math

import pytest

from oracle import scheduling as S
from paper_2109_01611_amd import scenarios

SIZES, BATCHES = list(scenarios.SIZES), list(scenarios.BATCHES)


# ------------------------------------------------------------------ derivative and curvature formulas

def test_three_point_derivatives_exact_on_parabolas_with_uneven_spacing():
    a, b, c = -1.75, 0.4, 3.0
    f = lambda x: a * x * x + b * x + c
    for x0, x1, x2 in [(0.0, 0.25, 1.0), (-2.0, 1.0, 1.5), (0.2, 0.4, 0.5)]:
        d1, d2 = S.three_point_derivatives(x0, f(x0), x1, f(x1), x2, f(x2))
        assert d1 == pytest.approx(2 * a * x1 + b, rel=1e-12)
        assert d2 == pytest.approx(2 * a, rel=1e-12)


def test_curvature_of_a_circle_arc_is_one_over_radius_and_positive_when_concave():
    R = 2.5
    xs = [-1.0 + 0.002 * i for i in range(1001)]
    upper = [math.sqrt(R * R - x * x) for x in xs]
    k = S.curvature(xs, upper)
    assert k[0] == 0.0 and k[-1] == 0.0
    for i in range(1, len(xs) - 1):
        assert k[i] == pytest.approx(1.0 / R, rel=1e-4)
    lower = [-v for v in upper]
    assert all(v == pytest.approx(-1.0 / R, rel=1e-4) for v in S.curvature(xs, lower)[1:-1])


def test_curvature_of_parabola_matches_closed_form_on_the_profiled_grid():
    a = 0.9
    xs = [s / 100.0 for s in SIZES]
    ys = [-a * x * x for x in xs]
    k = S.curvature(xs, ys)
    for i in range(1, len(xs) - 1):
        assert k[i] == pytest.approx(2 * a / (1 + 4 * a * a * xs[i] ** 2) ** 1.5, rel=1e-12)


# ------------------------------------------------------------------ knee

def test_knee_of_a_hockey_stick_is_the_break_point():
    for knee in (40, 50, 60, 80):
        rates = [10.0 * min(s, knee) + 0.5 * max(0, s - knee) for s in SIZES]
        assert S.max_efficient_partition(SIZES, rates) == knee


def test_knee_is_invariant_to_units_of_rate():
    rates = [100.0, 200.0, 250.0, 260.0, 270.0, 280.0]
    assert S.max_efficient_partition(SIZES, rates) == 50
    assert S.max_efficient_partition(SIZES, [7.5 * r + 3 for r in rates]) == 50


def test_linear_convex_and_flat_curves_have_no_knee():
    assert S.max_efficient_partition(SIZES, [3.0 * s for s in SIZES]) == 100
    assert S.max_efficient_partition(SIZES, [float(s * s) for s in SIZES]) == 100
    assert S.max_efficient_partition(SIZES, [5.0] * len(SIZES)) == 100
    assert S.max_efficient_partition([50, 100], [1.0, 2.0]) == 100


def test_ties_go_to_the_smaller_size():
    # identical bends (slope 3 -> 1) at 40 and 80 on an evenly spaced grid; every value exact in binary
    sizes = [20, 40, 60, 80, 100]
    rates = [0.0, 3.0, 4.0, 7.0, 8.0]
    k = S.curvature(S.normalised([float(s) for s in sizes]), S.normalised(rates))
    assert k[1] == k[3] > 0 > k[2]
    assert S.max_efficient_partition(sizes, rates) == 40


# ------------------------------------------------------------------ affordable rate

def test_affordable_rate_closed_form_for_affine_latency():
    alpha, beta = 1.0, 0.5                       # L(b) = 1 + 0.5 b ms: throughput rises with b
    row = [alpha + beta * b for b in BATCHES]
    for slo in (1.0, 3.0, 4.0, 10.0, 13.9, 34.0, 1000.0):
        rate, j = S.affordable_rate(row, BATCHES, slo)
        ok = [b for b in BATCHES if alpha + beta * b <= slo / 2]
        if not ok:
            assert (rate, j) == (0.0, -1)
        else:
            b = max(ok)
            assert BATCHES[j] == b and rate == pytest.approx(1000.0 * b / (alpha + beta * b), rel=1e-15)
            assert S.max_batch(row, BATCHES, slo) == j


def test_affordable_rate_takes_the_best_batch_not_the_largest():
    row = [1.0, 1.5, 2.0, 9.0, 40.0, 90.0]       # throughput peaks at b=4
    rate, j = S.affordable_rate(row, BATCHES, 1000.0)
    assert BATCHES[j] == 4 and rate == pytest.approx(2000.0)
    assert S.max_batch(row, BATCHES, 1000.0) == len(BATCHES) - 1


def test_interference_scales_latency():
    row = [1.0, 2.0, 4.0, 8.0, 16.0, 32.0]
    assert S.max_batch(row, BATCHES, 16.0, 0.0) == 3
    assert S.max_batch(row, BATCHES, 16.0, 0.01) == 2
    rate, j = S.affordable_rate(row, BATCHES, 16.0, 0.25)
    assert BATCHES[j] == 1 and rate == pytest.approx(1000.0 / 1.25)


def replay(rate, b, latency_ms, n_batches):
    """Event-by-event serving of regularly arriving requests in batches of b:
    a batch is dispatched when its last request has arrived and the gpu-let
    is free.  Returns the worst request latency in ms."""
    gap = 1000.0 / rate
    free_at, worst = 0.0, 0.0
    for k in range(n_batches):
        arrivals = [(k * b + i) * gap for i in range(b)]
        start = max(arrivals[-1], free_at)
        free_at = start + latency_ms
        worst = max(worst, free_at - arrivals[0])
    return worst


def test_replay_of_serving_at_the_affordable_rate_meets_the_slo_and_overload_does_not():
    row = [0.8 + 0.3 * b for b in BATCHES]
    for slo in (4.0, 8.0, 21.0):
        rate, j = S.affordable_rate(row, BATCHES, slo)
        b, lat = BATCHES[j], row[j]
        assert replay(rate, b, lat, 4000) <= slo
        assert replay(rate, b, lat, 4000) == pytest.approx(lat + (b - 1) * lat / b, rel=1e-9)
        assert replay(rate * 1.05, b, lat, 4000) > slo          # backlog grows without bound
        # the next larger batch size would break the budget even when the gpu-let keeps up
        if j + 1 < len(BATCHES):
            assert 2 * row[j + 1] > slo


def test_min_required_partition():
    rates = [100.0, 190.0, 230.0, 260.0, 300.0, 320.0]
    assert S.min_required_partition(SIZES, rates, 50.0) == 20
    assert S.min_required_partition(SIZES, rates, 100.0) == 20
    assert S.min_required_partition(SIZES, rates, 100.5) == 40
    assert S.min_required_partition(SIZES, rates, 261.0) == 80
    assert S.min_required_partition(SIZES, rates, 1000.0) == 100


def test_interference_matrix_is_the_linear_model_of_sec_4_4():
    c = [0.5, 0.25, 0.125, 1.0, -0.1]
    l2, mem = [0.2, 0.8], [0.4, 0.1]
    F = S.interference_matrix(c, l2, mem)
    assert F[0][1] == pytest.approx(0.5 * 0.2 + 0.25 * 0.8 + 0.125 * 0.4 + 1.0 * 0.1 - 0.1)
    assert F[1][0] == pytest.approx(0.5 * 0.8 + 0.25 * 0.2 + 0.125 * 0.1 + 1.0 * 0.4 - 0.1)
    assert S.interference_matrix([0, 0, 0, 0, -1.0], l2, mem) == [[0.0, 0.0], [0.0, 0.0]]


# ------------------------------------------------------------------ Algorithm 1: hand-worked cases

def scaling_table(per_image_ms, fixed_ms=0.0):
    """L(b, p) = fixed + per_image * b * 100 / p: latency inversely proportional to the share."""
    return [[fixed_ms + per_image_ms * b * 100.0 / p for b in BATCHES] for p in SIZES]


def knee_table(per_image_ms, knee):
    """Like scaling_table but shares beyond ``knee`` percent bring nothing."""
    return [[per_image_ms * b * 100.0 / min(p, knee) for b in BATCHES] for p in SIZES]


def test_one_small_model_gets_the_smallest_sufficient_gpulet():
    # 1 ms per image on the whole GPU, 5 ms on 20%: any batch fits, every size sustains 10*p req/s
    prob = S.Problem(SIZES, BATCHES, [scaling_table(1.0)], [150.0], [1000.0], 1)
    ok, entries = S.elastic_partitioning(prob)
    # affordable rate is linear in p: no knee, p_eff = 100; p_req = 20 (200 req/s >= 150)
    assert ok and entries == [(0, 20, 0, 0, 32, 150.0, 0.0)]


def test_rate_beyond_the_knee_is_served_by_several_knee_sized_gpulets():
    # knee at 40%: A(p) = 10*min(p, 40) req/s.  900 req/s -> 40% (400), 40% (400), then p_req=20 (100 left)
    prob = S.Problem(SIZES, BATCHES, [knee_table(1.0, 40)], [900.0], [1000.0], 2)
    ok, entries = S.elastic_partitioning(prob)
    assert ok
    # first pass splits GPU 0 into 40/60; the second pass takes the 60% leftover (best fit >= 40),
    # which sustains no more than 400 req/s; the last 100 req/s get a 20% gpu-let of GPU 1
    assert [(e[0], e[1], e[2]) for e in entries] == [(0, 40, 0), (0, 60, 1), (1, 20, 0)]
    assert [e[5] for e in entries] == pytest.approx([400.0, 400.0, 100.0])
    assert sum(e[5] for e in entries) == pytest.approx(900.0)


def test_models_are_taken_in_descending_rate_and_best_fit_reuses_leftovers():
    tabs = [scaling_table(1.0), scaling_table(1.0)]
    prob = S.Problem(SIZES, BATCHES, tabs, [150.0, 700.0], [1000.0, 1000.0], 1, merge=False)
    ok, entries = S.elastic_partitioning(prob)
    # model 1 (700 req/s) first: p_req = 80 -> split 80/20; model 0 (150) fits the 20% leftover
    assert ok and [(e[3], e[1], e[2]) for e in entries] == [(1, 80, 0), (0, 20, 1)]


def test_not_schedulable_when_gpulets_run_out():
    prob = S.Problem(SIZES, BATCHES, [scaling_table(1.0)], [1500.0], [1000.0], 1)
    ok, entries = S.elastic_partitioning(prob)
    assert not ok and sum(e[5] for e in entries) == pytest.approx(1000.0)
    prob.n_gpu = 2
    ok, entries = S.elastic_partitioning(prob)
    assert ok and sum(e[5] for e in entries) == pytest.approx(1500.0)


def test_slo_too_tight_for_any_batch_is_not_schedulable():
    prob = S.Problem(SIZES, BATCHES, [scaling_table(1.0)], [10.0], [1.9], 4)
    assert S.elastic_partitioning(prob) == (False, [])


def test_light_models_merge_onto_one_gpulet_by_time_sharing():
    # two models of 0.1 ms per image: L(1, 20%) = 0.5 ms each; at 100 req/s both share one 20% gpu-let
    tabs = [scaling_table(0.1), scaling_table(0.1)]
    prob = S.Problem(SIZES, BATCHES, tabs, [100.0, 100.0], [50.0, 50.0], 1)
    ok, entries = S.elastic_partitioning(prob)
    assert ok and [(e[0], e[1], e[2], e[3]) for e in entries] == [(0, 20, 0, 0), (0, 20, 0, 1)]
    # shortest round: one batch of 1 each, 0.5 + 0.5 ms; 0.1 requests arrive per round
    assert entries[0][6] == entries[1][6] == pytest.approx(1.0)
    assert [e[4] for e in entries] == [1, 1]
    prob.merge = False
    ok, entries = S.elastic_partitioning(prob)
    assert ok and [(e[1], e[2], e[3]) for e in entries] == [(20, 0, 0), (80, 1, 1)]


def test_merge_is_tried_even_when_no_free_gpulet_is_left():
    # whole GPUs only (one profiled size): the second model has no gpu-let to claim but time-shares the first
    tabs = [[[0.1 * b for b in BATCHES]], [[0.2 * b for b in BATCHES]]]
    prob = S.Problem([100], BATCHES, tabs, [100.0, 50.0], [50.0, 50.0], 1)
    ok, entries = S.elastic_partitioning(prob)
    assert ok and [(e[0], e[1], e[2], e[3], e[4]) for e in entries] == [(0, 100, 0, 0, 1), (0, 100, 0, 1, 1)]
    assert entries[0][6] == pytest.approx(0.1 + 0.2)
    prob.merge = False
    ok, entries = S.elastic_partitioning(prob)
    assert not ok and [e[3] for e in entries] == [0]
    # three models on one split GPU: the third has to share
    tabs = [scaling_table(0.1)] * 3
    prob = S.Problem(SIZES, BATCHES, tabs, [1500.0, 1200.0, 100.0], [1000.0] * 3, 1)
    ok, entries = S.elastic_partitioning(prob)
    assert ok and sorted(set((e[1], e[2]) for e in entries)) == [(20, 0), (80, 1)]
    check_schedule(prob, ok, entries)


def test_duty_cycle_is_the_least_fixed_point_of_the_round_length():
    # one model, L(b) = 1 + b ms on every size, 1500 req/s: b >= 1.5 * (1 + b) never holds up to 32 -> not sharable
    tab = [[1.0 + b for b in BATCHES] for _ in SIZES]
    prob = S.Problem(SIZES, BATCHES, [tab], [1500.0], [1000.0], 1)
    assert S.temporally_sharable(prob, 100, [(0, 1500.0)], lambda m: 0.0) is None
    # 800 req/s: b >= 0.8 * (1 + b) first holds at b = 4 (5 ms covers 4 requests); the iteration
    # walks 0 -> 2 (b=1) -> 3 (b=2) -> 5 (b=4) -> settles
    d, picks = S.temporally_sharable(prob, 100, [(0, 800.0)], lambda m: 0.0)
    assert (d, [BATCHES[j] for j in picks]) == (5.0, [4])
    # the same round breaks an SLO shorter than d + L
    prob.slo = [9.9]
    assert S.temporally_sharable(prob, 100, [(0, 800.0)], lambda m: 0.0) is None
    prob.slo = [10.0]
    assert S.temporally_sharable(prob, 100, [(0, 800.0)], lambda m: 0.0) is not None
    # a slowdown stretches every execution
    prob.slo = [1000.0]
    d, picks = S.temporally_sharable(prob, 100, [(0, 400.0)], lambda m: 0.5)
    # L' = 1.5 (1 + b): b >= 0.4 * 1.5 * (1 + b) = 0.6 + 0.6 b -> b >= 1.5 -> b = 2, d = 4.5
    assert (d, [BATCHES[j] for j in picks]) == (4.5, [2])


def replay_round_robin(members, duty_ms, rounds):
    """Event-by-event replay of time sharing: ``members`` = [(rate, batch, latency)],
    each with a fixed slot per round of ``duty_ms`` (slots back to back in list
    order).  A slot runs the requests that arrived since the model's previous
    slot began.  Returns per member (largest batch seen, worst request latency)."""
    out, offset = [], 0.0
    for rate, batch, lat in members:
        gap = 1000.0 / rate
        phase = 0.37 * gap                      # arrival phase, arbitrary
        worst_lat, worst_b = 0.0, 0
        nxt = 0                                 # index of the next request not yet served
        for k in range(rounds):
            start = offset + k * duty_ms
            n = int(math.floor((start - phase) / gap)) + 1 - nxt if start >= phase else 0
            if n > 0:
                first = phase + nxt * gap
                worst_lat = max(worst_lat, start + lat - first)
                worst_b = max(worst_b, n)
                nxt += n
        out.append((worst_b, worst_lat))
        offset += lat
    return out, offset


def test_replay_of_merged_gpulets_stays_within_batch_sizes_and_slos():
    seen = 0
    for seed in range(300):
        prob = random_problem(seed, 2 + seed % 4, 1 + seed % 3, False, True, load=0.08)
        ok, entries = S.elastic_partitioning(prob)
        groups = {}
        for e in entries:
            if e[6] > 0:
                groups.setdefault((e[0], e[2]), []).append(e)
        for (gpu, which), es in groups.items():
            size, d = es[0][1], es[0][6]
            members = [(e[5], e[4], prob.L[e[3]][SIZES.index(size)][BATCHES.index(e[4])]) for e in es]
            res, busy = replay_round_robin(members, d, 3000)
            assert busy <= d * (1 + 1e-12)
            for (worst_b, worst_lat), e in zip(res, es):
                assert worst_b <= e[4]
                assert worst_lat <= prob.slo[e[3]] * (1 + 1e-9)
            seen += 1
    assert seen > 30


def test_interference_refuses_a_neighbour_that_breaks_the_budget():
    # model 0 fills 80% with batch 32 exactly at its budget; any slowdown from a neighbour breaks it
    t0 = scaling_table(1.0)
    slo0 = 2 * t0[SIZES.index(80)][-1]
    tabs = [t0, scaling_table(0.1)]
    F = [[0.0, 0.2], [0.0, 0.0]]
    rates = [32 * 1000.0 / t0[SIZES.index(80)][-1], 100.0]
    prob = S.Problem(SIZES, BATCHES, tabs, rates, [slo0, 1000.0], 2, intf=F, merge=False)
    ok, entries = S.elastic_partitioning(prob)
    assert ok
    by_model = {e[3]: e for e in entries}
    assert by_model[0][:3] == (0, 80, 0)
    assert by_model[1][0] == 1                       # pushed to the other GPU
    prob.F = [[0.0, 0.0], [0.0, 0.0]]
    ok, entries = S.elastic_partitioning(prob)
    assert {e[3]: e for e in entries}[1][:3] == (0, 20, 1)


# ------------------------------------------------------------------ Algorithm 1: invariants on random scenarios

def check_schedule(prob, ok, entries):
    """Everything a valid schedule must satisfy under the latency budget."""
    by_gpulet = {}
    for gpu, size, which, m, b, r, d in entries:
        assert size in prob.sizes and b in prob.batches and r > 0
        by_gpulet.setdefault((gpu, which), {"size": size, "duty": d, "members": []})
        g = by_gpulet[(gpu, which)]
        assert g["size"] == size and g["duty"] == d
        g["members"].append((m, b, r))
    for gpu in set(k[0] for k in by_gpulet):
        parts = [v for k, v in by_gpulet.items() if k[0] == gpu]
        assert len(parts) <= 2 and sum(p["size"] for p in parts) <= 100
        assert 0 <= gpu < prob.n_gpu
    served = [0.0] * len(prob.rate)
    for (gpu, which), g in by_gpulet.items():
        other = by_gpulet.get((gpu, 1 - which))
        for m, b, r in g["members"]:
            served[m] += r
            f = max([prob.F[m][o[0]] for o in other["members"]]) if other else 0.0
            lat = prob.L[m][prob.sizes.index(g["size"])][prob.batches.index(b)] * (1 + f)
            if g["duty"] == 0.0:
                assert len(g["members"]) == 1
                assert lat <= prob.slo[m] / 2 * (1 + 1e-12)
                assert r <= 1000.0 * b / lat * (1 + 1e-12)
            else:
                assert g["duty"] + lat <= prob.slo[m] * (1 + 1e-12)
                assert b >= r * g["duty"] / 1000.0 * (1 - 1e-9)
        if g["duty"] > 0.0:
            total = 0.0
            for m, b, r in g["members"]:
                f = max([prob.F[m][o[0]] for o in other["members"]]) if other else 0.0
                total += prob.L[m][prob.sizes.index(g["size"])][prob.batches.index(b)] * (1 + f)
            assert total <= g["duty"] * (1 + 1e-12)
            assert len(set(m for m, _, _ in g["members"])) == len(g["members"])
    for m in range(len(prob.rate)):
        if ok:
            assert served[m] == pytest.approx(prob.rate[m], rel=1e-9, abs=1e-9)
        else:
            assert served[m] <= prob.rate[m] * (1 + 1e-9)


def random_problem(seed, n_models, n_gpu, with_intf, merge=True, load=1.5):
    from paper_2109_01611_amd import inputs
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
    return S.Problem(SIZES, BATCHES, tabs, rates, slos, n_gpu, intf=F, merge=merge)


@pytest.mark.parametrize("with_intf", [False, True])
@pytest.mark.parametrize("merge", [False, True])
def test_random_scenarios_produce_valid_schedules(with_intf, merge):
    n_ok = 0
    for seed in range(120):
        prob = random_problem(seed, 1 + seed % 5, 1 + (seed // 5) % 4, with_intf, merge)
        ok, entries = S.elastic_partitioning(prob)
        check_schedule(prob, ok, entries)
        n_ok += ok
    assert 10 < n_ok < 120          # the generator exercises both outcomes


def test_more_gpus_never_hurt():
    for seed in range(60):
        prev = False
        for n_gpu in (1, 2, 3, 4, 6):
            prob = random_problem(seed, 4, n_gpu, True)
            ok, _ = S.elastic_partitioning(prob)
            assert ok or not prev
            prev = ok


def test_schedule_is_deterministic_and_ignores_idle_models():
    prob = random_problem(7, 4, 3, True)
    a = S.elastic_partitioning(prob)
    assert a == S.elastic_partitioning(prob)
    prob.rate[2] = 0.0
    ok, entries = S.elastic_partitioning(prob)
    assert all(e[3] != 2 for e in entries)


def test_paper_tables():
    assert len(scenarios.rate_grid(5)) == 4 ** 5 - 1
    assert scenarios.rate_grid(2)[0] == [0.0, 200.0]
    assert scenarios.PAPER_SLO_MS == {"goo": 44.0, "le": 5.0, "res": 95.0, "ssd": 136.0, "vgg": 130.0}
    assert scenarios.PAPER_SCENARIOS["long-only"] == {"le": 0.0, "goo": 0.0, "res": 100.0, "ssd": 100.0, "vgg": 100.0}
    assert [sum(s.values()) for s in scenarios.PAPER_SCENARIOS.values()] == [250.0, 300.0, 400.0]
