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


# The whole GPU's L2 request rate (16 channels on each of 8 dies, one request per clock at 2.4 GHz) and
# HBM bandwidth: what solo-run counter totals are put in relation to.
L2_PEAK_REQ_PER_S = 128 * 2.4e9
HBM_PEAK_BYTES_PER_S = 8e12


def interference_utilisation(l2_requests, fetch_bytes, write_bytes, solo_ms, l2_peak=L2_PEAK_REQ_PER_S,
                             mem_peak=HBM_PEAK_BYTES_PER_S):
    """-> (L2 utilisation, memory-bandwidth utilisation) of one solo run from its counter totals."""
    l2, mem = c_double(), c_double()
    _check(lib.gpulet_interference_utilisation(l2_requests, fetch_bytes, write_bytes, solo_ms, l2_peak, mem_peak,
                                               byref(l2), byref(mem)), "gpulet_interference_utilisation")
    return l2.value, mem.value


def interference_factor(corun_ms, solo_ms):
    n = len(corun_ms)
    out = (c_double * n)()
    _check(lib.gpulet_interference_factor(_doubles(corun_ms), _doubles(solo_ms), n, out),
           "gpulet_interference_factor")
    return list(out)


def interference_split(keys):
    """-> (training indices, validation indices): 70 / 30 in the order of the seeded keys."""
    n = len(keys)
    order, n_train = (c_int * n)(), c_int()
    _check(lib.gpulet_interference_split(_doubles(keys), n, order, byref(n_train)), "gpulet_interference_split")
    return list(order[:n_train.value]), list(order[n_train.value:])


def interference_worst_slowdown(coef, features):
    out = c_double()
    _check(lib.gpulet_interference_worst_slowdown(_doubles(coef), _flat(features), len(features), byref(out)),
           "gpulet_interference_worst_slowdown")
    return out.value


def interference_overhead(factors, percentiles=(50.0, 90.0, 99.0, 100.0), threshold=0.18):
    """-> (overhead = factor - 1 at the percentiles (nearest rank), share of samples below ``threshold``)."""
    out, share = (c_double * len(percentiles))(), c_double()
    _check(lib.gpulet_interference_overhead(_doubles(factors), len(factors), _doubles(percentiles), len(percentiles),
                                            out, threshold, byref(share)), "gpulet_interference_overhead")
    return list(out), share.value


__all__ = ["affordable_rate", "rate_curve", "max_efficient_partition", "min_required_partition",
           "elastic_partitioning", "interference_fit", "interference_predict", "interference_error",
           "interference_utilisation", "interference_factor", "interference_split", "interference_worst_slowdown",
           "interference_overhead", "gpulet"]
