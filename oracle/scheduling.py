"""Plain-Python oracle of the scheduler side of gpu-lets (paper Sec. 4.3, Algorithm 1).

Test infrastructure only: tests and the smoke check may import this file, the
product never does.  It shares no code with the C++ scheduler in the library;
it follows the paper's procedure step by step in the paper's notation, in fp64
(Python floats), with plain loops.

What the paper fixes and what is a reading of it
------------------------------------------------
The paper prints no worked example of Algorithm 1 and leaves several steps
open, so the *outcome* of ``elastic_partitioning`` is "parity unpinned": it is
pinned only through invariants every valid schedule must satisfy and through
hand-worked tiny cases (see the tests).  The building blocks are pinned by
closed forms.  The readings taken here:

* Latency budget (Sec. 2.2).  A request violates its SLO when batch building
  time plus batch execution time exceed the SLO.  With batches of b built at
  rate r back to back, building takes b/r and execution L; the gpu-let keeps
  up iff L <= b/r, so at the highest sustainable rate r = b/L the worst
  request sees 2L.  Hence a batch size is admissible on a gpu-let iff
  L(b, p) + intf <= SLO/2 and the rate it then sustains is b / (L + intf).
  "L(k, size) <= SLO" in FindBestFit is read with this execution budget.
* Affordable rate of a gpu-let size (Sec. 4.3, Fig. 8): the largest sustained
  rate over admissible profiled batch sizes.
* Knee (MaxEfficientPartition): both axes of the affordable-rate curve are
  scaled to [0, 1]; at every interior profiled size the parabola through the
  point and its two neighbours gives y' and y''; the signed curvature is
  -y'' / (1 + y'^2)^(3/2) (positive where the curve bends towards the
  flat); p_eff is the size of largest curvature, the smaller size on ties,
  and the largest profiled size when no interior point bends that way.
* MinRequiredPartition: smallest profiled size whose affordable rate covers
  the rate still unassigned; the largest size if none does (the rest is
  handled by the next pass of the while loop).
* intf: a fractional slowdown F[victim][aggressor] >= 0 applied to L when the
  other gpu-let of the same GPU is occupied (largest value over the models
  there).  A placement is also refused when it would push a model already on
  the partner gpu-let over its own budget or below the rate assigned to it.
* Temporally sharable / Merge: models share a gpu-let round-robin.  A round
  of length d runs, for every model i, the smallest profiled batch size b_i
  that covers the requests arriving during d (at least the smallest profiled
  batch); busy(d) = sum_i L_i(b_i).  The duty cycle is the least d with
  busy(d) <= d (iterate d <- busy(d) from 0) and the set is sharable iff it
  exists within the profiled batch sizes and d + L_i(b_i) <= SLO_i for every
  i.  For a single model this reduces to the budget above.  Merge is also
  tried when no free gpu-let fits (the listing does not say what happens
  then); the model then offers the rate a gpu-let of p_ideal would have taken.
* Order: gpu-lets of equal size are visited by GPU index, then by position on
  the GPU; models of equal rate by index.
"""

TOL = 1e-12  # relative slack where a quantity equals a profiled batch size up to rounding


# --------------------------------------------------------------------------- rate curve

def sustained_rate(b, latency_ms):
    """Requests per second when batches of b run back to back at ``latency_ms`` each."""
    return 1000.0 * b / latency_ms


def max_batch(latency_row, batches, slo_ms, intf=0.0):
    """Index of the largest profiled batch size whose slowed-down latency fits
    the execution budget SLO/2, or -1.  ``latency_row[j]`` is L(batches[j], p)."""
    best = -1
    for j in range(len(batches)):
        if latency_row[j] * (1.0 + intf) <= 0.5 * slo_ms:
            best = j
    return best


def affordable_rate(latency_row, batches, slo_ms, intf=0.0):
    """(rate in req/s, batch index) a gpu-let sustains within the SLO: the best
    admissible profiled batch size; (0.0, -1) if none is admissible."""
    rate, arg = 0.0, -1
    for j in range(len(batches)):
        lat = latency_row[j] * (1.0 + intf)
        if lat <= 0.5 * slo_ms:
            r = sustained_rate(batches[j], lat)
            if r > rate:
                rate, arg = r, j
    return rate, arg


def rate_curve(table, batches, slo_ms):
    """Affordable rate for every profiled size; ``table[i][j]`` = L(batches[j], sizes[i])."""
    return [affordable_rate(row, batches, slo_ms)[0] for row in table]


# --------------------------------------------------------------------------- knee

def three_point_derivatives(x0, y0, x1, y1, x2, y2):
    """y' and y'' at x1 of the parabola through three points (x0 < x1 < x2)."""
    h1, h2 = x1 - x0, x2 - x1
    s1, s2 = (y1 - y0) / h1, (y2 - y1) / h2
    d1 = (h1 * s2 + h2 * s1) / (h1 + h2)
    d2 = 2.0 * (s2 - s1) / (h1 + h2)
    return d1, d2


def curvature(x, y):
    """Signed curvature -y''/(1+y'^2)^1.5 at the interior points of a sampled
    curve; the two end points get 0."""
    k = [0.0] * len(x)
    for i in range(1, len(x) - 1):
        d1, d2 = three_point_derivatives(x[i - 1], y[i - 1], x[i], y[i], x[i + 1], y[i + 1])
        k[i] = -d2 / (1.0 + d1 * d1) ** 1.5
    return k


def normalised(v):
    lo, hi = min(v), max(v)
    if hi == lo:
        return [0.0] * len(v)
    return [(e - lo) / (hi - lo) for e in v]


def max_efficient_partition(sizes, rates):
    """p_eff: the profiled size at the knee of the affordable-rate curve."""
    if len(sizes) < 3:
        return sizes[-1]
    k = curvature(normalised([float(s) for s in sizes]), normalised(rates))
    best, arg = 0.0, -1
    for i in range(1, len(sizes) - 1):
        if k[i] > best:
            best, arg = k[i], i
    return sizes[arg] if arg >= 0 else sizes[-1]


def min_required_partition(sizes, rates, rate):
    """p_req: the smallest profiled size whose affordable rate covers ``rate``."""
    for i in range(len(sizes)):
        if rates[i] >= rate:
            return sizes[i]
    return sizes[-1]


# --------------------------------------------------------------------------- interference model (Sec. 4.4)

def interference_matrix(c, l2, mem):
    """F[m1][m2] = c1*l2[m1] + c2*l2[m2] + c3*mem[m1] + c4*mem[m2] + c5, floored at 0."""
    n = len(l2)
    return [[max(0.0, c[0] * l2[a] + c[1] * l2[b] + c[2] * mem[a] + c[3] * mem[b] + c[4]) for b in range(n)]
            for a in range(n)]


# --------------------------------------------------------------------------- Algorithm 1

class Gpulet:
    """One gpu-let: ``size`` percent of GPU ``gpu``; ``which`` 0 for the first
    part of a split (or the whole GPU), 1 for the remainder.  ``alloc`` lists
    [model, batch, rate] in order of assignment; ``duty_ms`` is 0 while one
    model runs back to back and the cycle length once several share it."""

    def __init__(self, gpu, size, which):
        self.gpu, self.size, self.which = gpu, size, which
        self.alloc = []
        self.duty_ms = 0.0

    def key(self):
        return (self.size, self.gpu, self.which)


class Problem:
    def __init__(self, sizes, batches, tables, rates, slos, n_gpu, intf=None, merge=True):
        self.sizes, self.batches = list(sizes), list(batches)
        self.L = tables              # L[m][size index][batch index] in ms
        self.rate, self.slo = list(rates), list(slos)
        self.n_gpu, self.merge = n_gpu, merge
        n = len(self.rate)
        self.F = intf if intf is not None else [[0.0] * n for _ in range(n)]

    def row(self, m, size):
        return self.L[m][self.sizes.index(size)]


def _partner(gpus, g):
    parts = gpus[g.gpu]
    return parts[1 - g.which] if len(parts) == 2 else None


def _slowdown(prob, m, other):
    """Largest fractional slowdown the models on gpu-let ``other`` inflict on model m."""
    if other is None or not other.alloc:
        return 0.0
    return max(prob.F[m][a[0]] for a in other.alloc)


def _cycle_load(prob, size, members, f_of, d):
    """Batches one round of length d collects on a gpu-let of ``size``: per member
    the smallest profiled batch size covering the requests that arrive during d.
    Returns (batch indices, slowed-down latencies) or None past the profile."""
    picks, lats = [], []
    for m, r in members:
        need = r * d / 1000.0
        j = -1
        for jj in range(len(prob.batches)):
            if prob.batches[jj] >= need * (1.0 - TOL):
                j = jj
                break
        if j < 0:
            return None
        picks.append(j)
        lats.append(prob.row(m, size)[j] * (1.0 + f_of(m)))
    return picks, lats


def _cycle_feasible(prob, size, members, f_of, d):
    """Batch indices if ``members`` fit a duty cycle of d within their SLOs, else None."""
    load = _cycle_load(prob, size, members, f_of, d)
    if load is None:
        return None
    picks, lats = load
    total = 0.0
    for (m, r), lat in zip(members, lats):
        if d + lat > prob.slo[m]:
            return None
        total += lat
    return picks if total <= d else None


def temporally_sharable(prob, size, members, f_of):
    """Shortest duty cycle for ``members`` = [(model, rate)] time-sharing one
    gpu-let of ``size``: the least d with busy(d) <= d, found by iterating
    d <- busy(d) from 0, where busy(d) is the time to run every member's batch
    of one round.  Returns (d, batch indices), or None when the iteration
    leaves the profiled batch sizes, does not settle, or an SLO breaks."""
    d = 0.0
    for _ in range(len(members) * len(prob.batches) + 2):
        load = _cycle_load(prob, size, members, f_of, d)
        if load is None:
            return None
        busy = 0.0
        for lat in load[1]:
            busy += lat
        if busy <= d:
            picks = _cycle_feasible(prob, size, members, f_of, d)
            return (d, picks) if picks is not None else None
        d = busy
    return None


def _partner_still_fits(prob, gpus, g, m):
    """Would the models on the partner of gpu-let g stay within budget with m beside them?"""
    other = _partner(gpus, g)
    if other is None or not other.alloc:
        return True
    def f_of(v):
        return max([prob.F[v][m]] + [prob.F[v][a[0]] for a in g.alloc])
    members = [(a[0], a[2]) for a in other.alloc]
    if len(members) == 1 and other.duty_ms == 0.0:
        v, j, r = other.alloc[0][0], prob.batches.index(other.alloc[0][1]), other.alloc[0][2]
        lat = prob.row(v, other.size)[j] * (1.0 + f_of(v))
        return lat <= 0.5 * prob.slo[v] and sustained_rate(prob.batches[j], lat) >= r
    return _cycle_feasible(prob, other.size, members, f_of, other.duty_ms) is not None


def find_best_fit(prob, gpus, order_alloc, m, p_ideal, want):
    """FindBestFit of Algorithm 1 for model m: returns (gpu-let, batch, rate) after
    updating ``gpus`` / ``order_alloc``, or None when no remaining gpu-let fits."""
    remain = sorted([g for parts in gpus for g in parts if not g.alloc], key=Gpulet.key)
    chosen, b_idx, f = None, -1, 0.0
    for g in remain:
        if g.size < p_ideal:
            continue
        split = False
        if g.size == 100 and p_ideal < 100:          # Split
            gpus[g.gpu] = [Gpulet(g.gpu, p_ideal, 0), Gpulet(g.gpu, 100 - p_ideal, 1)]
            g, split = gpus[g.gpu][0], True
        f = _slowdown(prob, m, _partner(gpus, g))
        b_idx = max_batch(prob.row(m, g.size), prob.batches, prob.slo[m], f)
        if b_idx >= 0 and _partner_still_fits(prob, gpus, g, m):
            chosen = g
            break
        if split:
            gpus[g.gpu] = [Gpulet(g.gpu, 100, 0)]
    if chosen is not None:
        lat = prob.row(m, chosen.size)[b_idx] * (1.0 + f)
        take = min(want, sustained_rate(prob.batches[b_idx], lat))
    elif prob.merge:
        # no free gpu-let fits: time sharing is still tried, with the rate a
        # gpu-let of the ideal size would have taken
        take = min(want, affordable_rate(prob.row(m, p_ideal), prob.batches, prob.slo[m])[0])
        if take <= 0.0:
            return None
    else:
        return None

    if prob.merge:
        for a in order_alloc:                         # Merge through temporal sharing
            if any(e[0] == m for e in a.alloc):
                continue
            other = _partner(gpus, a)
            def f_of(v, other=other):
                return _slowdown(prob, v, other)
            members = [(e[0], e[2]) for e in a.alloc] + [(m, take)]
            res = temporally_sharable(prob, a.size, members, f_of)
            if res is None:
                continue
            # the partner of `a` must also survive m as a new neighbour
            if not _partner_still_fits(prob, gpus, a, m):
                continue
            d, picks = res
            a.alloc.append([m, 0, take])
            for e, j in zip(a.alloc, picks):
                e[1] = prob.batches[j]
            a.duty_ms = d
            if chosen is not None:
                parts = gpus[chosen.gpu]              # RevertSplit
                if len(parts) == 2 and not parts[0].alloc and not parts[1].alloc:
                    gpus[chosen.gpu] = [Gpulet(chosen.gpu, 100, 0)]
            return a, a.alloc[-1][1], take
    if chosen is None:
        return None

    chosen.alloc.append([m, prob.batches[b_idx], take])
    order_alloc.append(chosen)
    return chosen, prob.batches[b_idx], take


def elastic_partitioning(prob):
    """One scheduling period of Algorithm 1.  Returns (schedulable, entries)
    where entries lists (gpu, size, which, model, batch, rate, duty_ms) per model
    and gpu-let, gpu-lets in order of first allocation."""
    gpus = [[Gpulet(g, 100, 0)] for g in range(prob.n_gpu)]   # reset remain_gpulets
    order_alloc = []
    models = sorted(range(len(prob.rate)), key=lambda m: (-prob.rate[m], m))
    ok = True
    for m in models:
        remaining = prob.rate[m]
        if remaining <= 0.0:
            continue
        curve = rate_curve(prob.L[m], prob.batches, prob.slo[m])
        p_eff = max_efficient_partition(prob.sizes, curve)
        while remaining > 0.0:
            p_req = min_required_partition(prob.sizes, curve, remaining)
            p_ideal = min(p_eff, p_req)
            res = find_best_fit(prob, gpus, order_alloc, m, p_ideal, remaining)
            if res is None:
                ok = False
                break
            take = res[2]
            remaining = 0.0 if take >= remaining else remaining - take
        if not ok:
            break
    entries = []
    for g in order_alloc:
        for m, b, r in g.alloc:
            entries.append((g.gpu, g.size, g.which, m, b, r, g.duty_ms))
    return ok, entries


def gpus_used(entries):
    return len(set(e[0] for e in entries))
