// Interference model of co-located gpu-lets (paper Sec. 4.4): a linear model
// in the solo-run L2 and memory-bandwidth utilisation of victim and aggressor,
// fitted by least squares.  Host-only fp64 code.
#include <algorithm>
#include <cmath>
#include <vector>

#include "gpulet_sched.h"

namespace {

constexpr int NC = 5;  // c1..c4 and the constant c5

bool finite_all(const double *v, long long n) {
    if (!v) return false;
    for (long long i = 0; i < n; ++i)
        if (!std::isfinite(v[i])) return false;
    return true;
}

// Least squares through Householder QR of the n x 5 design matrix [features | 1].
// Returns false when a column is (numerically) dependent on the ones before it.
bool least_squares(const double *features, const double *y, int n, double *coef) {
    std::vector<double> a(static_cast<size_t>(n) * NC), b(y, y + n);
    double scale[NC];
    for (int i = 0; i < n; ++i) {
        for (int j = 0; j < 4; ++j) a[static_cast<size_t>(i) * NC + j] = features[static_cast<size_t>(i) * 4 + j];
        a[static_cast<size_t>(i) * NC + 4] = 1.0;
    }
    for (int j = 0; j < NC; ++j) {
        double s = 0.0;
        for (int i = 0; i < n; ++i) s += a[static_cast<size_t>(i) * NC + j] * a[static_cast<size_t>(i) * NC + j];
        scale[j] = std::sqrt(s);
    }
    double diag[NC];
    for (int k = 0; k < NC; ++k) {
        double norm = 0.0;
        for (int i = k; i < n; ++i) norm += a[static_cast<size_t>(i) * NC + k] * a[static_cast<size_t>(i) * NC + k];
        norm = std::sqrt(norm);
        if (!(norm > 1e-12 * scale[k]) || scale[k] == 0.0) return false;
        const double akk = a[static_cast<size_t>(k) * NC + k];
        const double alpha = akk > 0.0 ? -norm : norm;
        // v = x - alpha e1 stored in place; H = I - 2 v v^T / (v^T v)
        a[static_cast<size_t>(k) * NC + k] = akk - alpha;
        double vtv = 0.0;
        for (int i = k; i < n; ++i) vtv += a[static_cast<size_t>(i) * NC + k] * a[static_cast<size_t>(i) * NC + k];
        for (int j = k + 1; j < NC; ++j) {
            double dot = 0.0;
            for (int i = k; i < n; ++i) dot += a[static_cast<size_t>(i) * NC + k] * a[static_cast<size_t>(i) * NC + j];
            const double f = 2.0 * dot / vtv;
            for (int i = k; i < n; ++i) a[static_cast<size_t>(i) * NC + j] -= f * a[static_cast<size_t>(i) * NC + k];
        }
        double dot = 0.0;
        for (int i = k; i < n; ++i) dot += a[static_cast<size_t>(i) * NC + k] * b[i];
        const double f = 2.0 * dot / vtv;
        for (int i = k; i < n; ++i) b[i] -= f * a[static_cast<size_t>(i) * NC + k];
        diag[k] = alpha;
    }
    for (int k = NC - 1; k >= 0; --k) {  // back substitution with R (diagonal kept aside)
        double s = b[k];
        for (int j = k + 1; j < NC; ++j) s -= a[static_cast<size_t>(k) * NC + j] * coef[j];
        coef[k] = s / diag[k];
    }
    return true;
}

double model(const double *c, const double *f) { return c[0] * f[0] + c[1] * f[1] + c[2] * f[2] + c[3] * f[3] + c[4]; }

}  // namespace

extern "C" {

gpulet_status gpulet_interference_fit(const double *features, const double *factor, int n, double *coef) {
    if (!coef || n < NC || !finite_all(features, 4LL * n) || !finite_all(factor, n)) return GPULET_EINVAL;
    return least_squares(features, factor, n, coef) ? GPULET_OK : GPULET_EINVAL;
}

gpulet_status gpulet_interference_predict(const double *coef, const double *features, int n, double *factor) {
    if (!factor || n < 1 || !finite_all(coef, NC) || !finite_all(features, 4LL * n)) return GPULET_EINVAL;
    for (int i = 0; i < n; ++i) factor[i] = model(coef, features + 4LL * i);
    return GPULET_OK;
}

gpulet_status gpulet_interference_error(const double *coef, const double *features, const double *factor, int n,
                                        const double *q, int n_q, double *error_at_q) {
    if (!error_at_q || !q || n < 1 || n_q < 1 || !finite_all(coef, NC) || !finite_all(features, 4LL * n) ||
        !finite_all(factor, n))
        return GPULET_EINVAL;
    std::vector<double> err(n);
    for (int i = 0; i < n; ++i) {
        if (!(factor[i] > 0.0)) return GPULET_EINVAL;
        err[i] = std::fabs(model(coef, features + 4LL * i) - factor[i]) / factor[i];
    }
    std::sort(err.begin(), err.end());
    for (int k = 0; k < n_q; ++k) {
        if (!(q[k] > 0.0) || !(q[k] <= 100.0)) return GPULET_EINVAL;
        const int rank = static_cast<int>(std::ceil(q[k] / 100.0 * n));
        error_at_q[k] = err[std::max(0, rank - 1)];
    }
    return GPULET_OK;
}

gpulet_status gpulet_interference_utilisation(double l2_requests, double fetch_bytes, double write_bytes,
                                              double solo_ms, double l2_peak_requests_per_s,
                                              double mem_peak_bytes_per_s, double *l2_util, double *mem_util) {
    if (!l2_util || !mem_util) return GPULET_EINVAL;
    const double v[6] = {l2_requests, fetch_bytes, write_bytes, solo_ms, l2_peak_requests_per_s, mem_peak_bytes_per_s};
    if (!finite_all(v, 6)) return GPULET_EINVAL;
    if (l2_requests < 0.0 || fetch_bytes < 0.0 || write_bytes < 0.0 || !(solo_ms > 0.0) ||
        !(l2_peak_requests_per_s > 0.0) || !(mem_peak_bytes_per_s > 0.0))
        return GPULET_EINVAL;
    const double seconds = solo_ms * 1e-3;
    *l2_util = l2_requests / seconds / l2_peak_requests_per_s;
    *mem_util = (fetch_bytes + write_bytes) / seconds / mem_peak_bytes_per_s;
    return GPULET_OK;
}

gpulet_status gpulet_interference_factor(const double *corun_ms, const double *solo_ms, int n, double *factor) {
    if (!factor || n < 1 || !finite_all(corun_ms, n) || !finite_all(solo_ms, n)) return GPULET_EINVAL;
    for (int i = 0; i < n; ++i)
        if (!(corun_ms[i] > 0.0) || !(solo_ms[i] > 0.0)) return GPULET_EINVAL;
    for (int i = 0; i < n; ++i) factor[i] = corun_ms[i] / solo_ms[i];
    return GPULET_OK;
}

gpulet_status gpulet_interference_split(const double *key, int n, int *order, int *n_train) {
    if (!order || !n_train || n < 1 || !finite_all(key, n)) return GPULET_EINVAL;
    for (int i = 0; i < n; ++i) order[i] = i;
    std::stable_sort(order, order + n, [key](int a, int b) { return key[a] < key[b]; });
    *n_train = static_cast<int>((7LL * n) / 10);
    return GPULET_OK;
}

gpulet_status gpulet_interference_worst_slowdown(const double *coef, const double *features, int n,
                                                 double *slowdown) {
    if (!slowdown || n < 1 || !finite_all(coef, NC) || !finite_all(features, 4LL * n)) return GPULET_EINVAL;
    double worst = model(coef, features);
    for (int i = 1; i < n; ++i) worst = std::max(worst, model(coef, features + 4LL * i));
    *slowdown = std::max(0.0, worst - 1.0);
    return GPULET_OK;
}

gpulet_status gpulet_interference_overhead(const double *factor, int n, const double *q, int n_q,
                                           double *overhead_at_q, double threshold, double *share_below) {
    if (!overhead_at_q || !q || n < 1 || n_q < 1 || !finite_all(factor, n) || !std::isfinite(threshold))
        return GPULET_EINVAL;
    std::vector<double> over(factor, factor + n);
    for (double &o : over) o -= 1.0;
    std::sort(over.begin(), over.end());
    for (int k = 0; k < n_q; ++k) {
        if (!(q[k] > 0.0) || !(q[k] <= 100.0)) return GPULET_EINVAL;
        const int rank = static_cast<int>(std::ceil(q[k] / 100.0 * n));
        overhead_at_q[k] = over[std::max(0, rank - 1)];
    }
    if (share_below) {
        long long below = 0;
        for (double o : over) below += o < threshold ? 1 : 0;
        *share_below = static_cast<double>(below) / static_cast<double>(n);
    }
    return GPULET_OK;
}

}  // extern "C"
