/*
 * gpulet_sched.h - C ABI of the scheduler side of gpu-lets: host-only, fp64,
 * no GPU call anywhere in this header.
 *
 * Paper: arXiv 2109.01611, Sec. 4.3.  The scheduler consumes, per model, the
 * profiled latency L(b, p) of batch b on a gpu-let of p percent (Table 2), a
 * per-model SLO (Table 4) and an interference function, and each period maps
 * models to gpu-lets (Algorithm 1: ElasticPartitioning, FindBestFit, Split,
 * Merge, RevertSplit).  Its two helper curves are the affordable request rate
 * of a gpu-let size and the knee of that curve (MaxEfficientPartition, Fig. 8)
 * and the smallest size that covers a rate (MinRequiredPartition).
 *
 * Where the paper leaves a step open this library takes the following
 * readings (the same ones its test oracle takes, so that both can be compared
 * decision by decision):
 *   - Execution budget (Sec. 2.2: batch building time plus execution time
 *     must stay within the SLO).  A gpu-let that runs batches of b back to
 *     back at latency L sustains b/L requests per unit time and its worst
 *     request waits one building period plus one execution, 2L.  A batch size
 *     is admissible iff L(b, p) * (1 + f) <= SLO / 2, f being the fractional
 *     slowdown from the neighbour gpu-let.
 *   - Affordable rate of a size: the best sustained rate over admissible
 *     profiled batch sizes.
 *   - Knee: both axes scaled to [0, 1]; y' and y'' at each interior profiled
 *     size from the parabola through the point and its two neighbours;
 *     curvature -y'' / (1 + y'^2)^1.5; the size of largest positive curvature
 *     (the smaller size on ties), the largest size if there is none.
 *   - Temporal sharing (Merge): models share a gpu-let round-robin.  A round
 *     of length d runs, for every model i, the smallest profiled batch b_i
 *     covering the requests that arrive during d; busy(d) = sum_i L_i(b_i).
 *     The duty cycle is the least d with busy(d) <= d (iterate d <- busy(d)
 *     from 0); the models are sharable iff it exists within the profiled
 *     batch sizes and d + L_i(b_i) <= SLO_i for every i.  Merge is also tried
 *     when no free gpu-let fits; the model then offers the rate a gpu-let of
 *     the ideal size would have taken.
 *   - A placement is refused when it would push the models on the partner
 *     gpu-let of the same GPU over their budget or below their assigned rate.
 *   - Visiting order: gpu-lets by (size, gpu, position); models by
 *     (rate descending, index).
 *
 * All arrays are HOST memory owned by the caller and only read during the
 * call (outputs only written).  Rates are requests per second, times are
 * milliseconds, sizes are percent.  Calls are pure and thread safe.
 * Errors: GPULET_EINVAL for NULL pointers, non-positive counts, sizes or
 * batches that are not strictly ascending and positive, sizes that do not end
 * at 100, non-finite or non-positive latencies or SLOs, negative rates or
 * slowdowns; GPULET_ENOMEM when an output array is too small.
 */
#ifndef GPULET_SCHED_H
#define GPULET_SCHED_H

#include "gpulet.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Affordable rate of one gpu-let size (Sec. 4.3, the curve of Fig. 8).
 * latency_ms[j] = L(batch[j], p).  `slowdown` is the fraction f above (0 when
 * the gpu-let has no neighbour).  Writes the rate (0 if no batch size is
 * admissible) and the batch size that reaches it (0 if none).
 */
gpulet_status gpulet_affordable_rate(const int *batch, const double *latency_ms, int n_batch, double slo_ms,
                                     double slowdown, double *rate, int *best_batch);

/*
 * The whole curve: latency_ms is [n_size][n_batch] row-major, rate gets
 * n_size values, one per profiled size, without slowdown.
 */
gpulet_status gpulet_rate_curve(const int *batch, int n_batch, int n_size, const double *latency_ms,
                                double slo_ms, double *rate);

/*
 * MaxEfficientPartition (Sec. 4.3): p_eff = profiled size at the knee of the
 * affordable-rate curve.  `curvature` may be NULL; otherwise it receives
 * n_size values (0 at both ends).
 */
gpulet_status gpulet_max_efficient_partition(const int *size, const double *rate, int n_size, int *p_eff,
                                             double *curvature);

/*
 * MinRequiredPartition (Sec. 4.3): p_req = smallest profiled size whose
 * affordable rate is >= want, the largest size if none is.
 */
gpulet_status gpulet_min_required_partition(const int *size, const double *rate, int n_size, double want,
                                            int *p_req);

/* One model of a scheduling problem. */
typedef struct gpulet_sched_model {
    double rate;              /* incoming request rate, req/s (0 = idle this period) */
    double slo_ms;            /* Table 4 */
    const double *latency_ms; /* L(b, p): [n_size][n_batch] row-major */
} gpulet_sched_model;

/*
 * One scheduling period's input.  For every profiled size s < 100 the
 * remainder 100 - s must be profiled too (Split hands it back as a gpu-let).
 */
typedef struct gpulet_sched_problem {
    int n_model, n_size, n_batch, n_gpu;
    const int *size;                 /* ascending, last = 100 */
    const int *batch;                /* ascending */
    const gpulet_sched_model *model; /* n_model */
    const double *slowdown;          /* [n_model][n_model] row-major: [victim][aggressor] fraction, or NULL = 0 */
    int merge;                       /* non-zero: try temporal sharing (Merge) after every best-fit */
} gpulet_sched_problem;

/* One (gpu-let, model) assignment of the result. */
typedef struct gpulet_sched_entry {
    int gpu;        /* 0 .. n_gpu-1 */
    int size;       /* percent */
    int which;      /* 0 = first part of the split (or the whole GPU), 1 = the remainder */
    int model;
    int batch;      /* batch size the model runs with on this gpu-let */
    double rate;    /* share of the model's rate served here, req/s */
    double duty_ms; /* 0 when the model has the gpu-let to itself, else the duty cycle it shares */
} gpulet_sched_entry;

/*
 * ElasticPartitioning (Algorithm 1), one period.  Entries come out grouped by
 * gpu-let in order of first allocation, models within a gpu-let in order of
 * assignment.  *schedulable is 1 when every model's rate was placed; when it
 * is 0 the entries hold what had been placed when the gpu-lets ran out.
 * GPULET_ENOMEM if more than max_entries would be written (*n_entries then
 * holds the number needed).
 */
gpulet_status gpulet_elastic_partitioning(const gpulet_sched_problem *problem, gpulet_sched_entry *entries,
                                          int max_entries, int *n_entries, int *schedulable);

/* ------------------------------------------------------------------------
 * Interference model (Sec. 4.4):
 *   factor = c1*l2_1 + c2*l2_2 + c3*mem_1 + c4*mem_2 + c5
 * l2 / mem = L2 and memory-bandwidth utilisation of the victim (1) and the
 * aggressor (2) in their solo runs; factor = the victim's co-run latency over
 * its solo latency on the same gpu-let.  `features` is [n][4] row-major in
 * the order (l2_1, l2_2, mem_1, mem_2); `coef` is c1..c5.
 * ------------------------------------------------------------------------ */

/*
 * Ordinary least squares over n >= 5 samples (Householder QR).  GPULET_EINVAL
 * when values are not finite or the samples do not determine five
 * coefficients (a feature column that is constant or a combination of the
 * others).
 */
gpulet_status gpulet_interference_fit(const double *features, const double *factor, int n, double *coef);

/* factor[i] of the model for n feature rows. */
gpulet_status gpulet_interference_predict(const double *coef, const double *features, int n, double *factor);

/*
 * Relative prediction error |model - measured| / measured over n samples
 * (measured factors must be positive), reported at the percentiles q[0..n_q)
 * (each in (0, 100], nearest rank) as in the error CDF of Fig. 9.
 */
gpulet_status gpulet_interference_error(const double *coef, const double *features, const double *factor, int n,
                                        const double *q, int n_q, double *error_at_q);

/*
 * The two features of one solo run (Sec. 4.4: L2 utilisation and DRAM bandwidth
 * utilisation "measured in the solo run" of a model at a batch size on a gpu-let):
 *   l2_util  = l2_requests / seconds / l2_peak_requests_per_s
 *   mem_util = (fetch_bytes + write_bytes) / seconds / mem_peak_bytes_per_s
 * with seconds = solo_ms / 1000: the counters of the whole run over the latency
 * of that run, relative to what the whole GPU can do (the shared L2 and memory
 * are not partitioned, so the peaks are the GPU's, not the gpu-let's share).
 * Counter totals must be >= 0, solo_ms and the peaks > 0, everything finite.
 */
gpulet_status gpulet_interference_utilisation(double l2_requests, double fetch_bytes, double write_bytes,
                                              double solo_ms, double l2_peak_requests_per_s,
                                              double mem_peak_bytes_per_s, double *l2_util, double *mem_util);

/* factor[i] = corun_ms[i] / solo_ms[i] (both > 0): how much slower the victim ran next to its neighbour. */
gpulet_status gpulet_interference_factor(const double *corun_ms, const double *solo_ms, int n, double *factor);

/*
 * Training / validation split of n samples (Sec. 4.4: 1,750 of 2,500 samples
 * for training, 750 for validation, i.e. 70 / 30): the samples are ordered by
 * the caller's keys key[0..n) (one seeded uniform draw per sample; equal keys
 * keep their index order), the first *n_train = floor(7 n / 10) of that order
 * train, the rest validate.  order receives the n sample indices in that order.
 */
gpulet_status gpulet_interference_split(const double *key, int n, int *order, int *n_train);

/*
 * Entry of the scheduler's slowdown matrix for one (victim, aggressor) pair of
 * models: the largest predicted factor over the n feature rows given (every
 * profiled pair of batch sizes and every split), minus one, not below zero.
 */
gpulet_status gpulet_interference_worst_slowdown(const double *coef, const double *features, int n,
                                                 double *slowdown);

/*
 * Distribution of the measured overhead factor - 1 over n co-runs (Fig. 6):
 * its value at the percentiles q[0..n_q) (nearest rank, as everywhere in this
 * library) and the share of samples strictly below `threshold` (the paper
 * quotes 18 %).  share_below may be NULL.
 */
gpulet_status gpulet_interference_overhead(const double *factor, int n, const double *q, int n_q,
                                           double *overhead_at_q, double threshold, double *share_below);

#ifdef __cplusplus
}
#endif
#endif /* GPULET_SCHED_H */
