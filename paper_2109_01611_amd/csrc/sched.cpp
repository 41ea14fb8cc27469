// Scheduler side of gpu-lets (paper Sec. 4.3, Algorithm 1): affordable-rate
// curve, its knee, and one period of elastic partitioning.  Host-only fp64
// code; no GPU call.  Built without floating-point contraction so that every
// comparison sees plainly rounded IEEE results.
#include <algorithm>
#include <cmath>
#include <vector>

#include "gpulet_sched.h"

namespace {

constexpr double kBatchSlack = 1e-12;  // relative slack where rate * cycle equals a profiled batch up to rounding

bool ascending_positive(const int *v, int n) {
    if (!v || n < 1) return false;
    for (int i = 0; i < n; ++i)
        if (v[i] < 1 || (i && v[i] <= v[i - 1])) return false;
    return true;
}

bool positive_finite(const double *v, int n) {
    if (!v) return false;
    for (int i = 0; i < n; ++i)
        if (!(v[i] > 0.0) || !std::isfinite(v[i])) return false;
    return true;
}

double slowed(double latency_ms, double f) { return latency_ms * (1.0 + f); }
double per_second(int b, double latency_ms) { return 1000.0 * b / latency_ms; }

// Largest profiled batch within the execution budget; -1 if none.
int largest_admissible(const double *row, int n_batch, double slo_ms, double f) {
    int best = -1;
    for (int j = 0; j < n_batch; ++j)
        if (slowed(row[j], f) <= 0.5 * slo_ms) best = j;
    return best;
}

double best_rate(const int *batch, const double *row, int n_batch, double slo_ms, double f, int *arg) {
    double rate = 0.0;
    *arg = -1;
    for (int j = 0; j < n_batch; ++j) {
        const double lat = slowed(row[j], f);
        if (lat > 0.5 * slo_ms) continue;
        const double r = per_second(batch[j], lat);
        if (r > rate) { rate = r; *arg = j; }
    }
    return rate;
}

void unit_scale(const double *v, int n, std::vector<double> &out) {
    const double lo = *std::min_element(v, v + n), hi = *std::max_element(v, v + n);
    out.resize(n);
    for (int i = 0; i < n; ++i) out[i] = hi == lo ? 0.0 : (v[i] - lo) / (hi - lo);
}

int knee(const int *size, const double *rate, int n, double *curv_out) {
    std::vector<double> curv(n, 0.0);
    if (n >= 3) {
        std::vector<double> sz(n), x, y;
        for (int i = 0; i < n; ++i) sz[i] = static_cast<double>(size[i]);
        unit_scale(sz.data(), n, x);
        unit_scale(rate, n, y);
        for (int i = 1; i + 1 < n; ++i) {
            const double h1 = x[i] - x[i - 1], h2 = x[i + 1] - x[i];
            const double s1 = (y[i] - y[i - 1]) / h1, s2 = (y[i + 1] - y[i]) / h2;
            const double d1 = (h1 * s2 + h2 * s1) / (h1 + h2);
            const double d2 = 2.0 * (s2 - s1) / (h1 + h2);
            curv[i] = -d2 / std::pow(1.0 + d1 * d1, 1.5);
        }
    }
    if (curv_out) std::copy(curv.begin(), curv.end(), curv_out);
    int arg = -1;
    double best = 0.0;
    for (int i = 1; i + 1 < n; ++i)
        if (curv[i] > best) { best = curv[i]; arg = i; }
    return size[arg >= 0 ? arg : n - 1];
}

int smallest_covering(const int *size, const double *rate, int n, double want) {
    for (int i = 0; i < n; ++i)
        if (rate[i] >= want) return size[i];
    return size[n - 1];
}

// ---------------------------------------------------------------- one period of Algorithm 1

struct Member { int model, batch_idx; double rate; };

struct Slot {               // one gpu-let
    int size = 0;
    double duty_ms = 0.0;
    std::vector<Member> members;
    bool free() const { return members.empty(); }
};

struct Gpu {
    int parts = 1;          // 1: whole, 2: split into slot[0] and slot[1]
    Slot slot[2];
    void make_whole() { parts = 1; slot[0] = Slot(); slot[0].size = 100; slot[1] = Slot(); }
    void split(int p) { parts = 2; slot[0] = Slot(); slot[1] = Slot(); slot[0].size = p; slot[1].size = 100 - p; }
};

struct Ref { int gpu, which; };

class Period {
  public:
    explicit Period(const gpulet_sched_problem &p) : P(p), gpus(p.n_gpu) {
        for (auto &g : gpus) g.make_whole();
    }

    bool run() {
        std::vector<int> order(P.n_model);
        for (int m = 0; m < P.n_model; ++m) order[m] = m;
        std::stable_sort(order.begin(), order.end(),
                         [&](int a, int b) { return P.model[a].rate > P.model[b].rate; });
        std::vector<double> curve(P.n_size);
        for (int m : order) {
            double remaining = P.model[m].rate;
            if (!(remaining > 0.0)) continue;
            for (int i = 0; i < P.n_size; ++i) {
                int arg;
                curve[i] = best_rate(P.batch, row(m, i), P.n_batch, P.model[m].slo_ms, 0.0, &arg);
            }
            const int p_eff = knee(P.size, curve.data(), P.n_size, nullptr);
            while (remaining > 0.0) {
                const int p_req = smallest_covering(P.size, curve.data(), P.n_size, remaining);
                double took;
                if (!best_fit(m, std::min(p_eff, p_req), remaining, &took)) return false;
                remaining = took >= remaining ? 0.0 : remaining - took;
            }
        }
        return true;
    }

    int count() const {
        int n = 0;
        for (const Ref &r : allocated) n += static_cast<int>(gpus[r.gpu].slot[r.which].members.size());
        return n;
    }

    void emit(gpulet_sched_entry *out) const {
        for (const Ref &r : allocated) {
            const Slot &s = gpus[r.gpu].slot[r.which];
            for (const Member &mb : s.members)
                *out++ = gpulet_sched_entry{r.gpu, s.size, r.which, mb.model, P.batch[mb.batch_idx], mb.rate,
                                            s.duty_ms};
        }
    }

  private:
    const gpulet_sched_problem &P;
    std::vector<Gpu> gpus;
    std::vector<Ref> allocated;   // gpu-lets in order of first allocation

    int size_index(int size) const {
        return static_cast<int>(std::find(P.size, P.size + P.n_size, size) - P.size);
    }
    const double *row(int m, int size_idx) const { return P.model[m].latency_ms + size_idx * P.n_batch; }
    double F(int victim, int aggressor) const {
        return P.slowdown ? P.slowdown[victim * P.n_model + aggressor] : 0.0;
    }
    const Slot *partner(Ref r) const {
        return gpus[r.gpu].parts == 2 ? &gpus[r.gpu].slot[1 - r.which] : nullptr;
    }
    // Worst slowdown of model v from the models on `s`, and from `extra` if >= 0.
    double slowdown_from(int v, const Slot *s, int extra = -1) const {
        double f = extra >= 0 ? F(v, extra) : 0.0;
        if (s)
            for (const Member &mb : s->members) f = std::max(f, F(v, mb.model));
        return f;
    }

    // One round of length d on a gpu-let of `size`: per member the smallest profiled batch covering
    // the requests that arrive during d, and its slowed-down latency.  `neigh`/`extra` say who slows
    // the members down.  False when a member needs more than the largest profiled batch.
    bool round_load(const std::vector<Member> &who, int size, double d, const Slot *neigh, int extra,
                    std::vector<int> *picks, std::vector<double> *lats) const {
        const int si = size_index(size);
        picks->clear();
        lats->clear();
        for (const Member &mb : who) {
            const double need = mb.rate * d / 1000.0;
            int j = 0;
            while (j < P.n_batch && !(P.batch[j] >= need * (1.0 - kBatchSlack))) ++j;
            if (j == P.n_batch) return false;
            picks->push_back(j);
            lats->push_back(slowed(row(mb.model, si)[j], slowdown_from(mb.model, neigh, extra)));
        }
        return true;
    }

    // Does a duty cycle of d hold every member's batch and every member's SLO?
    bool cycle_fits(const std::vector<Member> &who, int size, double d, const Slot *neigh, int extra,
                    std::vector<int> *picks) const {
        std::vector<double> lats;
        if (!round_load(who, size, d, neigh, extra, picks, &lats)) return false;
        double busy = 0.0;
        for (size_t i = 0; i < who.size(); ++i) {
            if (d + lats[i] > P.model[who[i].model].slo_ms) return false;
            busy += lats[i];
        }
        return busy <= d;
    }

    // Least d with busy(d) <= d, by iterating d <- busy(d) from 0; then the SLO test at that d.
    bool shortest_cycle(const std::vector<Member> &who, int size, const Slot *neigh, double *d_out,
                        std::vector<int> *picks) const {
        std::vector<double> lats;
        double d = 0.0;
        const int limit = static_cast<int>(who.size()) * P.n_batch + 2;
        for (int it = 0; it < limit; ++it) {
            if (!round_load(who, size, d, neigh, -1, picks, &lats)) return false;
            double busy = 0.0;
            for (double l : lats) busy += l;
            if (busy <= d) {
                *d_out = d;
                return cycle_fits(who, size, d, neigh, -1, picks);
            }
            d = busy;
        }
        return false;
    }

    // Do the models on the partner of `r` survive model m arriving on `r`?
    bool partner_survives(Ref r, int m) const {
        const Slot *other = partner(r);
        if (!other || other->free()) return true;
        const Slot *mine = &gpus[r.gpu].slot[r.which];
        if (other->members.size() == 1 && other->duty_ms == 0.0) {
            const Member &mb = other->members[0];
            const double lat = slowed(row(mb.model, size_index(other->size))[mb.batch_idx],
                                      slowdown_from(mb.model, mine, m));
            return lat <= 0.5 * P.model[mb.model].slo_ms && per_second(P.batch[mb.batch_idx], lat) >= mb.rate;
        }
        std::vector<int> picks;
        return cycle_fits(other->members, other->size, other->duty_ms, mine, m, &picks);
    }

    bool try_merge(int m, double take) {
        std::vector<int> picks;
        for (const Ref &r : allocated) {
            Slot &host = gpus[r.gpu].slot[r.which];
            bool has_m = false;
            for (const Member &mb : host.members) has_m |= mb.model == m;
            if (has_m) continue;
            std::vector<Member> who = host.members;
            who.push_back(Member{m, -1, take});
            double d;
            if (!shortest_cycle(who, host.size, partner(r), &d, &picks)) continue;
            if (!partner_survives(r, m)) continue;
            for (size_t i = 0; i < who.size(); ++i) who[i].batch_idx = picks[i];
            host.members = who;
            host.duty_ms = d;
            return true;
        }
        return false;
    }

    bool best_fit(int m, int p_ideal, double want, double *took) {
        // Ascending (size, gpu, position) over free gpu-lets without building a list: for every
        // profiled size from p_ideal up, scan the GPUs in order.
        Ref chosen{-1, 0};
        int b_idx = -1;
        double f = 0.0;
        bool did_split = false;
        for (int si = 0; si < P.n_size && chosen.gpu < 0; ++si) {
            const int size = P.size[si];
            if (size < p_ideal) continue;
            for (int g = 0; g < P.n_gpu && chosen.gpu < 0; ++g) {
                for (int w = 0; w < gpus[g].parts && chosen.gpu < 0; ++w) {
                    if (gpus[g].slot[w].size != size || !gpus[g].slot[w].free()) continue;
                    Ref r{g, w};
                    did_split = false;
                    if (size == 100 && p_ideal < 100) {
                        gpus[g].split(p_ideal);
                        did_split = true;
                    }
                    const Slot &s = gpus[g].slot[r.which];
                    f = slowdown_from(m, partner(r));
                    b_idx = largest_admissible(row(m, size_index(s.size)), P.n_batch, P.model[m].slo_ms, f);
                    if (b_idx >= 0 && partner_survives(r, m)) {
                        chosen = r;
                    } else if (did_split) {
                        gpus[g].make_whole();
                    }
                }
            }
        }
        if (chosen.gpu < 0) {
            // No free gpu-let fits: time sharing is still tried, with the rate a gpu-let of the
            // ideal size would have taken.
            if (!P.merge) return false;
            int arg;
            const double ideal = best_rate(P.batch, row(m, size_index(p_ideal)), P.n_batch, P.model[m].slo_ms,
                                           0.0, &arg);
            *took = std::min(want, ideal);
            return *took > 0.0 && try_merge(m, *took);
        }
        Slot &s = gpus[chosen.gpu].slot[chosen.which];
        const double lat = slowed(row(m, size_index(s.size))[b_idx], f);
        const double take = std::min(want, per_second(P.batch[b_idx], lat));
        *took = take;
        if (P.merge && try_merge(m, take)) {
            Gpu &g = gpus[chosen.gpu];   // RevertSplit
            if (g.parts == 2 && g.slot[0].free() && g.slot[1].free()) g.make_whole();
            return true;
        }
        s.members.push_back(Member{m, b_idx, take});
        allocated.push_back(chosen);
        return true;
    }
};

bool valid_problem(const gpulet_sched_problem *p) {
    if (!p || p->n_model < 1 || p->n_gpu < 1 || !p->model) return false;
    if (!ascending_positive(p->size, p->n_size) || !ascending_positive(p->batch, p->n_batch)) return false;
    if (p->size[p->n_size - 1] != 100) return false;
    for (int i = 0; i + 1 < p->n_size; ++i)
        if (std::find(p->size, p->size + p->n_size, 100 - p->size[i]) == p->size + p->n_size) return false;
    for (int m = 0; m < p->n_model; ++m) {
        const gpulet_sched_model &md = p->model[m];
        if (!(md.rate >= 0.0) || !std::isfinite(md.rate) || !(md.slo_ms > 0.0) || !std::isfinite(md.slo_ms))
            return false;
        if (!positive_finite(md.latency_ms, p->n_size * p->n_batch)) return false;
    }
    if (p->slowdown)
        for (int i = 0; i < p->n_model * p->n_model; ++i)
            if (!(p->slowdown[i] >= 0.0) || !std::isfinite(p->slowdown[i])) return false;
    return true;
}

}  // namespace

extern "C" {

gpulet_status gpulet_affordable_rate(const int *batch, const double *latency_ms, int n_batch, double slo_ms,
                                     double slowdown, double *rate, int *best_batch) {
    if (!rate || !best_batch || !ascending_positive(batch, n_batch) || !positive_finite(latency_ms, n_batch))
        return GPULET_EINVAL;
    if (!(slo_ms > 0.0) || !std::isfinite(slo_ms) || !(slowdown >= 0.0) || !std::isfinite(slowdown))
        return GPULET_EINVAL;
    int arg;
    *rate = best_rate(batch, latency_ms, n_batch, slo_ms, slowdown, &arg);
    *best_batch = arg >= 0 ? batch[arg] : 0;
    return GPULET_OK;
}

gpulet_status gpulet_rate_curve(const int *batch, int n_batch, int n_size, const double *latency_ms,
                                double slo_ms, double *rate) {
    if (!rate || n_size < 1 || !ascending_positive(batch, n_batch)) return GPULET_EINVAL;
    if (!positive_finite(latency_ms, n_size * n_batch) || !(slo_ms > 0.0) || !std::isfinite(slo_ms))
        return GPULET_EINVAL;
    for (int i = 0; i < n_size; ++i) {
        int arg;
        rate[i] = best_rate(batch, latency_ms + i * n_batch, n_batch, slo_ms, 0.0, &arg);
    }
    return GPULET_OK;
}

gpulet_status gpulet_max_efficient_partition(const int *size, const double *rate, int n_size, int *p_eff,
                                             double *curvature) {
    if (!p_eff || !rate || !ascending_positive(size, n_size)) return GPULET_EINVAL;
    for (int i = 0; i < n_size; ++i)
        if (!(rate[i] >= 0.0) || !std::isfinite(rate[i])) return GPULET_EINVAL;
    *p_eff = knee(size, rate, n_size, curvature);
    return GPULET_OK;
}

gpulet_status gpulet_min_required_partition(const int *size, const double *rate, int n_size, double want,
                                            int *p_req) {
    if (!p_req || !rate || !ascending_positive(size, n_size) || !(want >= 0.0)) return GPULET_EINVAL;
    *p_req = smallest_covering(size, rate, n_size, want);
    return GPULET_OK;
}

gpulet_status gpulet_elastic_partitioning(const gpulet_sched_problem *problem, gpulet_sched_entry *entries,
                                          int max_entries, int *n_entries, int *schedulable) {
    if (!n_entries || !schedulable || max_entries < 0 || (max_entries > 0 && !entries)) return GPULET_EINVAL;
    if (!valid_problem(problem)) return GPULET_EINVAL;
    Period period(*problem);
    *schedulable = period.run() ? 1 : 0;
    *n_entries = period.count();
    if (*n_entries > max_entries) return GPULET_ENOMEM;
    period.emit(entries);
    return GPULET_OK;
}

}  // extern "C"
