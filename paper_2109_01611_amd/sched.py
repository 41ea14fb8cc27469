"""Binding of the scheduler calls of ``libgpulet.so`` (``include/gpulet_sched.h``):
affordable-rate curve, MaxEfficientPartition, MinRequiredPartition and one
period of ElasticPartitioning (paper Sec. 4.3, Algorithm 1).

Argument marshalling only; every decision is taken inside the library.
"""

import ctypes
from ctypes import byref, c_double, c_int

from . import gpulet
from .gpulet import SchedEntry, SchedModel, SchedProblem, _check, lib


def _ints(v):
    return (c_int * len(v))(*[int(e) for e in v])


def _doubles(v):
    return (c_double * len(v))(*[float(e) for e in v])


def _flat(table):
    return _doubles([e for row in table for e in row])


def affordable_rate(batches, latency_row, slo_ms, slowdown=0.0):
    """-> (rate in req/s, batch size reaching it; 0 if no batch size is admissible)."""
    rate, best = c_double(), c_int()
    _check(lib.gpulet_affordable_rate(_ints(batches), _doubles(latency_row), len(batches), slo_ms, slowdown,
                                      byref(rate), byref(best)), "gpulet_affordable_rate")
    return rate.value, best.value


def rate_curve(batches, table, slo_ms):
    """Affordable rate per profiled size; ``table[i][j]`` = L(batches[j], sizes[i]) in ms."""
    out = (c_double * len(table))()
    _check(lib.gpulet_rate_curve(_ints(batches), len(batches), len(table), _flat(table), slo_ms, out),
           "gpulet_rate_curve")
    return list(out)


def max_efficient_partition(sizes, rates, with_curvature=False):
    p_eff = c_int()
    curv = (c_double * len(sizes))()
    _check(lib.gpulet_max_efficient_partition(_ints(sizes), _doubles(rates), len(sizes), byref(p_eff), curv),
           "gpulet_max_efficient_partition")
    return (p_eff.value, list(curv)) if with_curvature else p_eff.value


def min_required_partition(sizes, rates, want):
    p_req = c_int()
    _check(lib.gpulet_min_required_partition(_ints(sizes), _doubles(rates), len(sizes), want, byref(p_req)),
           "gpulet_min_required_partition")
    return p_req.value


def elastic_partitioning(sizes, batches, tables, rates, slos, n_gpu, slowdown=None, merge=True,
                         max_entries=None):
    """One scheduling period.  ``tables[m][i][j]`` = L_m(batches[j], sizes[i]) in ms,
    ``slowdown[victim][aggressor]`` a fraction.  Returns (schedulable, entries)
    with entries as (gpu, size, which, model, batch, rate, duty_ms) tuples."""
    n_model = len(rates)
    keep = [_flat(t) for t in tables]
    models = (SchedModel * n_model)()
    for m in range(n_model):
        models[m].rate, models[m].slo_ms = float(rates[m]), float(slos[m])
        models[m].latency_ms = ctypes.cast(keep[m], ctypes.POINTER(c_double))
    sz, bt = _ints(sizes), _ints(batches)
    sd = _flat(slowdown) if slowdown is not None else None
    prob = SchedProblem(n_model, len(sizes), len(batches), n_gpu, sz, bt, models,
                        ctypes.cast(sd, ctypes.POINTER(c_double)) if sd is not None else None, 1 if merge else 0)
    cap = max_entries if max_entries is not None else 2 * n_gpu * max(1, n_model) + 8
    entries = (SchedEntry * max(cap, 1))()
    n, ok = c_int(), c_int()
    _check(lib.gpulet_elastic_partitioning(byref(prob), entries, cap, byref(n), byref(ok)),
           "gpulet_elastic_partitioning")
    return bool(ok.value), [(e.gpu, e.size, e.which, e.model, e.batch, e.rate, e.duty_ms)
                            for e in entries[:n.value]]


def interference_fit(features, factors):
    """Least-squares c1..c5 of the interference model; ``features`` rows are
    (l2_victim, l2_aggressor, mem_victim, mem_aggressor)."""
    n = len(factors)
    coef = (c_double * 5)()
    _check(lib.gpulet_interference_fit(_flat(features), _doubles(factors), n, coef), "gpulet_interference_fit")
    return list(coef)


def interference_predict(coef, features):
    n = len(features)
    out = (c_double * n)()
    _check(lib.gpulet_interference_predict(_doubles(coef), _flat(features), n, out), "gpulet_interference_predict")
    return list(out)


def interference_error(coef, features, factors, percentiles=(90.0, 95.0)):
    """Relative prediction error at the given percentiles (nearest rank)."""
    n = len(factors)
    out = (c_double * len(percentiles))()
    _check(lib.gpulet_interference_error(_doubles(coef), _flat(features), _doubles(factors), n,
                                         _doubles(percentiles), len(percentiles), out),
           "gpulet_interference_error")
    return list(out)


__all__ = ["affordable_rate", "rate_curve", "max_efficient_partition", "min_required_partition",
           "elastic_partitioning", "interference_fit", "interference_predict", "interference_error", "gpulet"]
