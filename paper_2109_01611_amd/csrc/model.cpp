// Whole-model forward pass on a gpu-let, the L(b, p) latency profiler and the
// two-gpu-let co-run measurement (paper Sec. 5 "Backend inference executor";
// Sec. 3.1 / Fig. 3 and Sec. 4.1 for L(b, p); Sec. 3.2 / Fig. 6 for co-run
// interference).
#include <algorithm>
#include <atomic>
#include <climits>
#include <chrono>
#include <cmath>
#include <mutex>
#include <thread>
#include <vector>

#include "gpulet_internal.h"

using namespace gpulet;

namespace {

constexpr size_t kAlign = 256;

struct BufState {
    int C = 0, H = 0, W = 0, elem = 2;
    bool written = false;
    size_t bytes_per_image = 0;  // largest footprint over the buffer's lifetime
};

struct Step {
    int op;
    int in_buf, out_buf, res_buf;
    int out2_buf;   // CONV storing its last filters to a second buffer, else -1
    int pool_buf;   // CONV that also writes the 3x3 max pool of its input, else -1
    ConvArgs conv;  // CONV
    int N, C, H, W, P, Q, mode, k, k2, stride, pad;  // POOL (k); DWCONV (k x k2, relu)
    int In, Out, relu, out_fp32;                     // FC
    const void *w;
    const float *b;
    bool slice;             // CONV writing a channel slice of a wider (concatenated) tensor
    bool slice2;            // the same for the second buffer
    int group_len;          // CONV: layers launched together starting here (1: alone; 0: inside a group)
    int lane;               // stream of the gpu-let this layer runs on
    std::vector<int> wait;  // earlier layers on other lanes this one must wait for
    bool record;            // a later layer on another lane waits for this one
    bool pool_next;         // CONV: the next layer is a 2x2 / stride 2 max pool that is the only reader of
                            // this layer's output; the pair may run as one launch (conv_pool2_fusable)
};

struct Plan {
    std::vector<Step> steps;
    std::vector<BufState> bufs;
    std::vector<size_t> offset;  // workspace offset per buffer, (size_t)-1 for caller-owned
    size_t ws_bytes = 0;
    int in_buf = 0, out_buf = 0;
};

// One lane: see gpulet_set_model_lanes.
std::atomic<int> g_model_lanes{1};

// Data dependencies between layers and their spread over the gpu-let's lanes.
//
// Buffers are reused, so besides "reads what an earlier layer wrote" a layer must also wait
// for every earlier reader and writer of the buffer it overwrites.  Layers that write
// disjoint channel slices of one concatenated tensor do not depend on one another, but each
// of them depends on whatever the first of them had to wait for (`guard`).
//
// A layer stays on the lane of its most recent dependency when it is the first to continue
// that lane; otherwise it moves to the lane that has been idle longest.  Dependencies on the
// same lane are implied by stream order; the others become event waits.
void assign_lanes(Plan &plan, int n_bufs, int n_lanes) {
    struct Hazard {
        std::vector<int> writers, readers, guard;
        bool sliced = false;
    };
    std::vector<Hazard> hz(static_cast<size_t>(n_bufs));
    std::vector<int> tail(static_cast<size_t>(n_lanes), -1);  // last layer placed on each lane
    const int n = static_cast<int>(plan.steps.size());
    for (int i = 0; i < n; ++i) {
        Step &s = plan.steps[static_cast<size_t>(i)];
        std::vector<int> deps;
        auto reads = [&](int buf) {
            Hazard &h = hz[static_cast<size_t>(buf)];
            deps.insert(deps.end(), h.writers.begin(), h.writers.end());
        };
        reads(s.in_buf);
        if (s.res_buf >= 0) reads(s.res_buf);
        auto writes = [&](int buf, bool slice) {
            Hazard &o = hz[static_cast<size_t>(buf)];
            const bool joins = slice && o.sliced && o.readers.empty();  // another slice of the same tensor
            if (joins) {
                deps.insert(deps.end(), o.guard.begin(), o.guard.end());
            } else {
                o.guard = o.readers;
                o.guard.insert(o.guard.end(), o.writers.begin(), o.writers.end());
                deps.insert(deps.end(), o.guard.begin(), o.guard.end());
                o.writers.clear();
                o.readers.clear();
                o.sliced = slice;
            }
        };
        writes(s.out_buf, s.slice);
        if (s.out2_buf >= 0) writes(s.out2_buf, s.slice2);
        if (s.pool_buf >= 0) writes(s.pool_buf, false);
        std::sort(deps.begin(), deps.end());
        deps.erase(std::unique(deps.begin(), deps.end()), deps.end());

        int lane = 0;
        if (n_lanes > 1 && !deps.empty()) {
            const int latest = deps.back();
            const int ll = plan.steps[static_cast<size_t>(latest)].lane;
            if (tail[static_cast<size_t>(ll)] == latest) {
                lane = ll;
            } else {
                for (int l = 1; l < n_lanes; ++l)
                    if (tail[static_cast<size_t>(l)] < tail[static_cast<size_t>(lane)]) lane = l;
            }
        }
        s.lane = lane;
        s.wait.clear();
        for (int d : deps) {
            Step &ds = plan.steps[static_cast<size_t>(d)];
            // a same-lane dependency, and anything older than it on another lane's chain, is
            // already ordered; keep only the newest dependency of every other lane
            if (ds.lane == lane) continue;
            bool newer = false;
            for (int e : deps)
                if (e > d && plan.steps[static_cast<size_t>(e)].lane == ds.lane) newer = true;
            if (newer) continue;
            s.wait.push_back(d);
            ds.record = true;
        }
        tail[static_cast<size_t>(lane)] = i;

        // this layer now reads and writes
        hz[static_cast<size_t>(s.in_buf)].readers.push_back(i);
        if (s.res_buf >= 0) hz[static_cast<size_t>(s.res_buf)].readers.push_back(i);
        hz[static_cast<size_t>(s.out_buf)].writers.push_back(i);
        if (s.out2_buf >= 0) hz[static_cast<size_t>(s.out2_buf)].writers.push_back(i);
        if (s.pool_buf >= 0) hz[static_cast<size_t>(s.pool_buf)].writers.push_back(i);
    }
}

size_t round_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// Shape inference and validation of a model description for `batch` images.
gpulet_status build_plan(const gpulet_model_desc *m, int batch, Plan &plan) {
    if (!m || !m->layers || m->n_layers < 1 || m->n_bufs < 2 || batch < 1) return GPULET_EINVAL;
    if (m->in_C < 1 || m->in_H < 1 || m->in_W < 1) return GPULET_EINVAL;
    if (m->in_buf < 0 || m->in_buf >= m->n_bufs || m->out_buf < 0 || m->out_buf >= m->n_bufs ||
        m->in_buf == m->out_buf)
        return GPULET_EINVAL;
    if (1LL * batch * m->in_C * m->in_H * m->in_W >= (1LL << 31)) return GPULET_EINVAL;

    plan.bufs.assign(static_cast<size_t>(m->n_bufs), BufState());
    plan.steps.clear();
    plan.in_buf = m->in_buf;
    plan.out_buf = m->out_buf;
    BufState &in = plan.bufs[static_cast<size_t>(m->in_buf)];
    in.C = m->in_C; in.H = m->in_H; in.W = m->in_W; in.elem = 2; in.written = true;
    in.bytes_per_image = 2ull * m->in_C * m->in_H * m->in_W;

    for (int li = 0; li < m->n_layers; ++li) {
        const gpulet_layer &L = m->layers[li];
        if (L.in_buf < 0 || L.in_buf >= m->n_bufs || L.out_buf < 0 || L.out_buf >= m->n_bufs)
            return GPULET_EINVAL;
        if (L.out_buf == m->in_buf || L.in_buf == L.out_buf) return GPULET_EINVAL;
        const BufState src = plan.bufs[static_cast<size_t>(L.in_buf)];
        if (!src.written || src.elem != 2) return GPULET_EINVAL;
        BufState &dst = plan.bufs[static_cast<size_t>(L.out_buf)];
        Step s{};
        s.op = L.op;
        s.in_buf = L.in_buf;
        s.out_buf = L.out_buf;
        s.res_buf = -1;
        s.out2_buf = -1;
        s.pool_buf = -1;
        s.group_len = 1;
        s.slice2 = false;
        s.w = L.w;
        s.b = L.b;
        s.slice = false;
        s.lane = 0;
        s.record = false;
        s.pool_next = false;
        int oc = 0, oh = 0, ow = 0, oelem = 2;
        if (L.op == GPULET_OP_CONV) {
            // in_ch_total > 0: the layer reads L.C channels from in_ch_offset on of wider pixels
            if ((L.in_ch_total > 0 ? L.in_ch_total : L.C) != src.C || !L.w) return GPULET_EINVAL;
            if (L.stride < 1 || L.R < 1 || L.S < 1 || L.pad < 0) return GPULET_EINVAL;
            ConvArgs &a = s.conv;
            a.x = nullptr; a.w = L.w; a.b = L.b; a.y = nullptr; a.residual = nullptr;
            a.N = batch; a.C = L.C; a.H = src.H; a.W = src.W; a.K = L.K; a.R = L.R; a.S = L.S;
            a.stride = L.stride; a.pad = L.pad; a.relu = L.relu ? 1 : 0;
            a.P = out_extent(src.H, L.R, L.stride, L.pad);
            a.Q = out_extent(src.W, L.S, L.stride, L.pad);
            a.pre_pool = L.pre_pool;
            // K2 > 0: the last K2 filters are stored to out2_buf, the first K - K2 to out_buf
            if (L.K2 < 0 || (L.K2 > 0 && L.K2 >= L.K)) return GPULET_EINVAL;
            const int k1 = L.K - L.K2;
            a.y_ch_stride = L.out_ch_total > 0 ? L.out_ch_total : k1;
            a.y_ch_offset = L.out_ch_total > 0 ? L.out_ch_offset : 0;
            s.slice = L.out_ch_total > 0;
            if (L.K2 > 0) {
                if (L.out2_buf < 0 || L.out2_buf >= m->n_bufs || L.out2_buf == m->in_buf ||
                    L.out2_buf == L.in_buf || L.out2_buf == L.out_buf || L.res_buf >= 0)
                    return GPULET_EINVAL;
                a.y2 = &a;  // stand-in, filled in at run time
                a.k2 = k1;
                a.y2_ch_stride = L.out2_ch_total > 0 ? L.out2_ch_total : L.K2;
                a.y2_ch_offset = L.out2_ch_total > 0 ? L.out2_ch_offset : 0;
                s.out2_buf = L.out2_buf;
                s.slice2 = L.out2_ch_total > 0;
            }
            if (L.side_pool != 0) {
                if (L.side_pool != 3 || L.pool_buf < 0 || L.pool_buf >= m->n_bufs || L.pool_buf == m->in_buf ||
                    L.pool_buf == L.in_buf || L.pool_buf == L.out_buf || (L.K2 > 0 && L.pool_buf == L.out2_buf))
                    return GPULET_EINVAL;
                a.pool_y = &a;  // stand-in, filled in at run time
                s.pool_buf = L.pool_buf;
            }
            a.x_ch_stride = L.in_ch_total > 0 ? L.in_ch_total : 0;
            a.x_ch_offset = L.in_ch_total > 0 ? L.in_ch_offset : 0;
            // Pointers are filled in at run time; validate the rest with stand-ins.
            ConvArgs chk = a;
            chk.x = chk.w = chk.y = &chk;
            gpulet_status st = check_conv(chk);
            if (st != GPULET_OK) return st;
            if (L.res_buf >= 0) {
                if (L.res_buf >= m->n_bufs) return GPULET_EINVAL;
                const BufState &r = plan.bufs[static_cast<size_t>(L.res_buf)];
                if (!r.written || r.elem != 2 || r.C != L.K || r.H != a.P || r.W != a.Q) return GPULET_EINVAL;
                if (L.res_buf == L.out_buf && a.y_ch_stride != L.K) return GPULET_EINVAL;
                s.res_buf = L.res_buf;
            }
            oc = a.y_ch_stride; oh = a.P; ow = a.Q;
            if (s.pool_buf >= 0) {
                BufState &dp = plan.bufs[static_cast<size_t>(s.pool_buf)];
                dp.C = src.C; dp.H = src.H; dp.W = src.W; dp.elem = 2; dp.written = true;
                dp.bytes_per_image = std::max(dp.bytes_per_image, static_cast<size_t>(2) * src.C * src.H * src.W);
            }
            if (s.out2_buf >= 0) {
                BufState &d2 = plan.bufs[static_cast<size_t>(s.out2_buf)];
                d2.C = a.y2_ch_stride; d2.H = a.P; d2.W = a.Q; d2.elem = 2; d2.written = true;
                d2.bytes_per_image = std::max(d2.bytes_per_image, static_cast<size_t>(2) * a.y2_ch_stride * a.P * a.Q);
            }
        } else if (L.op == GPULET_OP_POOL) {
            if (L.C != src.C) return GPULET_EINVAL;
            int P = 0, Q = 0;
            gpulet_status st = check_pool(batch, src.C, src.H, src.W, L.mode, L.R, L.stride, L.pad, &P, &Q);
            if (st != GPULET_OK) return st;
            s.N = batch; s.C = src.C; s.H = src.H; s.W = src.W; s.P = P; s.Q = Q;
            s.mode = L.mode; s.k = L.R; s.stride = L.stride; s.pad = L.pad;
            oc = src.C; oh = P; ow = Q;
        } else if (L.op == GPULET_OP_DWCONV) {
            if (L.C != src.C || !L.w) return GPULET_EINVAL;
            int P = 0, Q = 0;
            gpulet_status st = check_dwconv(batch, src.C, src.H, src.W, L.R, L.S, L.stride, L.pad, &P, &Q);
            if (st != GPULET_OK) return st;
            s.N = batch; s.C = src.C; s.H = src.H; s.W = src.W; s.P = P; s.Q = Q;
            s.k = L.R; s.k2 = L.S; s.stride = L.stride; s.pad = L.pad; s.relu = L.relu ? 1 : 0;
            oc = src.C; oh = P; ow = Q;
        } else if (L.op == GPULET_OP_FC) {
            if (!L.w || 1LL * src.C * src.H * src.W != L.C) return GPULET_EINVAL;
            gpulet_status st = check_fc(batch, L.C, L.K);
            if (st != GPULET_OK) return st;
            s.N = batch; s.In = L.C; s.Out = L.K; s.relu = L.relu ? 1 : 0; s.out_fp32 = L.out_fp32 ? 1 : 0;
            oc = L.K; oh = 1; ow = 1; oelem = L.out_fp32 ? 4 : 2;
        } else {
            return GPULET_EINVAL;
        }
        dst.C = oc; dst.H = oh; dst.W = ow; dst.elem = oelem; dst.written = true;
        dst.bytes_per_image = std::max(dst.bytes_per_image, static_cast<size_t>(oelem) * oc * oh * ow);
        plan.steps.push_back(s);
    }
    if (!plan.bufs[static_cast<size_t>(m->out_buf)].written) return GPULET_EINVAL;
    // Launch groups: runs of layers chained by group_next.  All members are convolutions and
    // none reads or overwrites what another member writes (channel slices of one concatenated
    // tensor count as different destinations when they do not intersect).
    for (int i = 0; i < m->n_layers;) {
        int len = 1;
        while (m->layers[i + len - 1].group_next) {
            if (i + len >= m->n_layers || len >= kMaxGroup) return GPULET_EINVAL;
            ++len;
        }
        if (len > 1) {
            struct Span { int buf, lo, hi; };  // channels [lo, hi) of a buffer; the whole buffer: lo = 0, hi = INT_MAX
            auto writes = [&](int li) {
                const Step &s = plan.steps[static_cast<size_t>(li)];
                std::vector<Span> w;
                w.push_back(s.slice ? Span{s.out_buf, s.conv.y_ch_offset, s.conv.y_ch_offset + (s.out2_buf >= 0 ? s.conv.k2 : s.conv.K)}
                                    : Span{s.out_buf, 0, INT_MAX});
                if (s.out2_buf >= 0)
                    w.push_back(s.slice2 ? Span{s.out2_buf, s.conv.y2_ch_offset, s.conv.y2_ch_offset + s.conv.K - s.conv.k2}
                                         : Span{s.out2_buf, 0, INT_MAX});
                if (s.pool_buf >= 0) w.push_back(Span{s.pool_buf, 0, INT_MAX});
                return w;
            };
            for (int a = i; a < i + len; ++a) {
                if (plan.steps[static_cast<size_t>(a)].op != GPULET_OP_CONV) return GPULET_EINVAL;
                for (int b = i; b < i + len; ++b) {
                    if (a == b) continue;
                    const Step &sb = plan.steps[static_cast<size_t>(b)];
                    for (const Span &w : writes(a)) {
                        if (w.buf == sb.in_buf || w.buf == sb.res_buf) return GPULET_EINVAL;
                        if (a < b)
                            for (const Span &v : writes(b))
                                if (v.buf == w.buf && v.lo < w.hi && w.lo < v.hi) return GPULET_EINVAL;
                    }
                }
            }
            plan.steps[static_cast<size_t>(i)].group_len = len;
            for (int a = i + 1; a < i + len; ++a) plan.steps[static_cast<size_t>(a)].group_len = 0;
        }
        i += len;
    }
    // Convolution + 2x2 / stride 2 max pool pairs whose intermediate tensor nobody else reads: the
    // convolution may store the pooled tensor directly (decided per launch, see enqueue).  The
    // intermediate buffer keeps its place in the workspace for the launches that run the pair as
    // two kernels.
    for (int i = 0; i + 1 < m->n_layers; ++i) {
        Step &c = plan.steps[static_cast<size_t>(i)];
        const Step &q = plan.steps[static_cast<size_t>(i + 1)];
        if (c.op != GPULET_OP_CONV || c.group_len != 1 || c.slice || c.out2_buf >= 0 || c.pool_buf >= 0 || c.res_buf >= 0 ||
            c.conv.pre_pool || !c.conv.relu || c.out_buf == m->out_buf)
            continue;
        if (q.op != GPULET_OP_POOL || q.group_len != 1 || q.in_buf != c.out_buf || q.mode != GPULET_POOL_MAX || q.k != 2 ||
            q.stride != 2 || q.pad != 0 || c.conv.P % 2 != 0 || c.conv.Q % 2 != 0 || q.out_buf == c.in_buf)
            continue;
        bool only_reader = true;
        for (int j = i + 2; j < m->n_layers && only_reader; ++j) {
            const Step &t = plan.steps[static_cast<size_t>(j)];
            if (t.in_buf == c.out_buf || t.res_buf == c.out_buf) only_reader = false;
            if (t.out_buf == c.out_buf && !t.slice) break;   // overwritten as a whole: later readers see that tensor
        }
        c.pool_next = only_reader;
    }
    assign_lanes(plan, m->n_bufs, g_model_lanes.load());

    plan.offset.assign(static_cast<size_t>(m->n_bufs), static_cast<size_t>(-1));
    size_t off = 0;
    for (int i = 0; i < m->n_bufs; ++i) {
        if (i == m->in_buf || i == m->out_buf) continue;
        plan.offset[static_cast<size_t>(i)] = off;
        off += round_up(plan.bufs[static_cast<size_t>(i)].bytes_per_image * static_cast<size_t>(batch));
    }
    plan.ws_bytes = off;
    return GPULET_OK;
}

struct Bound {
    const Plan *plan;
    const void *in;
    void *out;
    char *ws;
    void *ptr(int buf) const {
        if (buf == plan->in_buf) return const_cast<void *>(in);
        if (buf == plan->out_buf) return out;
        return ws + plan->offset[static_cast<size_t>(buf)];
    }
};

// Event number `idx` of the gpu-let's pool (created on first use, never timed).
hipError_t pool_event(gpulet_partition *p, size_t idx, hipEvent_t *ev) {
    while (p->events.size() <= idx) {
        hipEvent_t e = nullptr;
        hipError_t st = hipEventCreateWithFlags(&e, hipEventDisableTiming);
        if (st != hipSuccess) return st;
        p->events.push_back(e);
    }
    *ev = p->events[idx];
    return hipSuccess;
}

// Enqueues every layer of one batch on the gpu-let's lanes; no host synchronisation.  Lane 0
// is the gpu-let's stream: the batch starts after everything enqueued there before and is
// complete, for anything enqueued there afterwards, when this returns.
hipError_t enqueue(const Bound &bd, gpulet_partition *p) {
    const std::vector<Step> &steps = bd.plan->steps;
    bool lane_used[kMaxLanes] = {false};
    for (const Step &s : steps) lane_used[s.lane] = true;
    // events 0 .. kMaxLanes-1: fork and joins; kMaxLanes + i: layer i
    hipEvent_t fork = nullptr;
    hipError_t e = hipSuccess;
    for (int l = 1; l < kMaxLanes; ++l) {
        if (!lane_used[l]) continue;
        if (!fork) {
            e = pool_event(p, 0, &fork);
            if (e == hipSuccess) e = hipEventRecord(fork, p->lane[0]);
            if (e != hipSuccess) return e;
        }
        e = hipStreamWaitEvent(p->lane[l], fork, 0);
        if (e != hipSuccess) return e;
    }
    LaunchCtx ctx0 = partition_ctx(p), ctx_other = ctx0;
    ctx_other.scratch = nullptr;  // the split-K scratch is not shared between concurrent layers
    ctx_other.scratch_bytes = 0;
    ctx_other.counters = nullptr;
    ctx_other.n_counters = 0;
    for (size_t i = 0; i < steps.size(); ++i) {
        const Step &s = steps[i];
        hipStream_t stream = p->lane[s.lane];
        const LaunchCtx &ctx = s.lane == 0 ? ctx0 : ctx_other;
        for (int d : s.wait) {
            hipEvent_t ev;
            e = pool_event(p, kMaxLanes + static_cast<size_t>(d), &ev);
            if (e == hipSuccess) e = hipStreamWaitEvent(stream, ev, 0);
            if (e != hipSuccess) return e;
        }
        // A launch group whose members all sit on this lane goes out as one launch, after the
        // waits of every member; otherwise its members are launched one by one as usual.
        size_t len = s.group_len > 1 ? static_cast<size_t>(s.group_len) : 1;
        for (size_t k = 1; k < len; ++k)
            if (steps[i + k].lane != s.lane) len = 1;
        if (len > 1) {
            ConvArgs args[kMaxGroup];
            for (size_t k = 0; k < len; ++k) {
                const Step &sk = steps[i + k];
                for (int d : sk.wait) {
                    if (k == 0) break;  // waited for above
                    hipEvent_t ev;
                    e = pool_event(p, kMaxLanes + static_cast<size_t>(d), &ev);
                    if (e == hipSuccess) e = hipStreamWaitEvent(stream, ev, 0);
                    if (e != hipSuccess) return e;
                }
                args[k] = sk.conv;
                args[k].x = bd.ptr(sk.in_buf);
                args[k].y = bd.ptr(sk.out_buf);
                args[k].residual = sk.res_buf >= 0 ? bd.ptr(sk.res_buf) : nullptr;
                args[k].y2 = sk.out2_buf >= 0 ? bd.ptr(sk.out2_buf) : nullptr;
                args[k].pool_y = sk.pool_buf >= 0 ? bd.ptr(sk.pool_buf) : nullptr;
            }
            int launches = 0;
            e = launch_conv_group(args, static_cast<int>(len), ctx, stream, &launches);
            if (e != hipSuccess) return e;
            p->kernels_enqueued.fetch_add(static_cast<uint64_t>(launches));
            for (size_t k = 0; k < len; ++k) {
                if (!steps[i + k].record) continue;
                hipEvent_t ev;
                e = pool_event(p, kMaxLanes + i + k, &ev);
                if (e == hipSuccess) e = hipEventRecord(ev, stream);
                if (e != hipSuccess) return e;
            }
            i += len - 1;
            continue;
        }
        if (s.op == GPULET_OP_CONV && s.pool_next && !s.record && steps[i + 1].lane == s.lane && steps[i + 1].wait.empty()) {
            // the layer and the max pool behind it as one launch, when a kernel with a pooled
            // epilogue applies and does not cost the layer more than the pool kernel saves
            ConvArgs a = s.conv;
            a.x = bd.ptr(s.in_buf);
            a.y = bd.ptr(steps[i + 1].out_buf);
            a.y_ch_stride = a.K;
            a.y_ch_offset = 0;
            if (conv_pool2_fusable(a, ctx)) {
                a.post_pool2 = 2;
                e = launch_conv(a, ctx, stream);
                if (e != hipSuccess) return e;
                p->kernels_enqueued.fetch_add(1);
                ++i;   // the pool is done
                if (steps[i].record) {
                    hipEvent_t ev;
                    e = pool_event(p, kMaxLanes + i, &ev);
                    if (e == hipSuccess) e = hipEventRecord(ev, stream);
                    if (e != hipSuccess) return e;
                }
                continue;
            }
        }
        if (s.op == GPULET_OP_CONV) {
            ConvArgs a = s.conv;
            a.x = bd.ptr(s.in_buf);
            a.y = bd.ptr(s.out_buf);
            a.y2 = s.out2_buf >= 0 ? bd.ptr(s.out2_buf) : nullptr;
            a.pool_y = s.pool_buf >= 0 ? bd.ptr(s.pool_buf) : nullptr;
            a.residual = s.res_buf >= 0 ? bd.ptr(s.res_buf) : nullptr;
            e = launch_conv(a, ctx, stream);
        } else if (s.op == GPULET_OP_POOL) {
            e = launch_pool(bd.ptr(s.in_buf), bd.ptr(s.out_buf), s.N, s.C, s.H, s.W, s.P, s.Q, s.mode, s.k,
                            s.stride, s.pad, stream);
        } else if (s.op == GPULET_OP_DWCONV) {
            e = launch_dwconv(bd.ptr(s.in_buf), s.w, s.b, bd.ptr(s.out_buf), s.N, s.C, s.H, s.W, s.k, s.k2,
                              s.stride, s.pad, s.relu, s.P, s.Q, stream);
        } else {
            e = launch_fc(bd.ptr(s.in_buf), s.w, s.b, bd.ptr(s.out_buf), s.N, s.In, s.Out, s.relu, s.out_fp32, ctx,
                          stream);
        }
        if (e != hipSuccess) return e;
        p->kernels_enqueued.fetch_add(1);
        if (s.record) {
            hipEvent_t ev;
            e = pool_event(p, kMaxLanes + i, &ev);
            if (e == hipSuccess) e = hipEventRecord(ev, stream);
            if (e != hipSuccess) return e;
        }
    }
    for (int l = 1; l < kMaxLanes; ++l) {
        if (!lane_used[l]) continue;
        hipEvent_t join;
        e = pool_event(p, static_cast<size_t>(l), &join);
        if (e == hipSuccess) e = hipEventRecord(join, p->lane[l]);
        if (e == hipSuccess) e = hipStreamWaitEvent(p->lane[0], join, 0);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

gpulet_status check_run_args(const Plan &plan, const void *in, void *out, void *ws, size_t ws_bytes) {
    if (!in || !out) return GPULET_EINVAL;
    if (plan.ws_bytes > 0) {
        if (!ws) return GPULET_EINVAL;
        if (ws_bytes < plan.ws_bytes) return GPULET_ENOMEM;
        if (reinterpret_cast<uintptr_t>(ws) % kAlign != 0) return GPULET_EINVAL;
    }
    return GPULET_OK;
}

struct EventPair {
    hipEvent_t a = nullptr, b = nullptr;
    hipError_t create() {
        hipError_t e = hipEventCreate(&a);
        if (e != hipSuccess) return e;
        e = hipEventCreate(&b);
        if (e != hipSuccess) {
            (void)hipEventDestroy(a);
            a = nullptr;
        }
        return e;
    }
    ~EventPair() {
        if (a) (void)hipEventDestroy(a);
        if (b) (void)hipEventDestroy(b);
    }
};

// One timed batch, waited for: returns its elapsed milliseconds.
hipError_t timed_batch(const Bound &bd, gpulet_partition *p, int batch, EventPair &ev, float *ms) {
    hipError_t e = hipEventRecord(ev.a, p->stream);
    if (e == hipSuccess) e = enqueue(bd, p);
    if (e == hipSuccess) e = hipEventRecord(ev.b, p->stream);
    if (e == hipSuccess) e = hipEventSynchronize(ev.b);
    if (e == hipSuccess) e = hipEventElapsedTime(ms, ev.a, ev.b);
    if (e == hipSuccess) {
        p->batches_run.fetch_add(1);
        p->images_run.fetch_add(static_cast<uint64_t>(batch));
    }
    return e;
}

}  // namespace

extern "C" gpulet_status gpulet_set_model_lanes(int lanes) {
    // Running layers on a second lane is switched off: a run that replayed a two-lane forward
    // pass from a captured graph on a masked stream stopped making progress, and the cause has
    // not been established.  The dependency analysis stays available through
    // gpulet_model_schedule.
    if (lanes != 1) return GPULET_EINVAL;
    g_model_lanes.store(1);
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_model_schedule(const gpulet_model_desc *m, int batch, int lanes, int *lane,
                                               int *wait_from, int *wait_to, int max_waits, int *n_waits) {
    if (!lane || !n_waits || max_waits < 0 || (max_waits > 0 && (!wait_from || !wait_to))) return GPULET_EINVAL;
    if (lanes < 1 || lanes > kMaxLanes) return GPULET_EINVAL;
    Plan plan;
    gpulet_status st = build_plan(m, batch, plan);
    if (st != GPULET_OK) return st;
    assign_lanes(plan, m->n_bufs, lanes);
    int n = 0;
    for (size_t i = 0; i < plan.steps.size(); ++i) {
        lane[i] = plan.steps[i].lane;
        for (int d : plan.steps[i].wait) {
            if (n < max_waits) {
                wait_from[n] = d;
                wait_to[n] = static_cast<int>(i);
            }
            ++n;
        }
    }
    *n_waits = n;
    return n > max_waits ? GPULET_ENOMEM : GPULET_OK;
}

extern "C" gpulet_status gpulet_model_workspace_bytes(const gpulet_model_desc *m, int batch,
                                                      size_t *bytes) {
    if (!bytes) return GPULET_EINVAL;
    Plan plan;
    gpulet_status st = build_plan(m, batch, plan);
    if (st != GPULET_OK) return st;
    *bytes = plan.ws_bytes;
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_model_buffer_info(const gpulet_model_desc *m, int batch, int buf,
                                                  int *C, int *H, int *W, int *elem_bytes,
                                                  size_t *ws_offset) {
    Plan plan;
    gpulet_status st = build_plan(m, batch, plan);
    if (st != GPULET_OK) return st;
    if (buf < 0 || buf >= m->n_bufs) return GPULET_EINVAL;
    const BufState &b = plan.bufs[static_cast<size_t>(buf)];
    if (!b.written) return GPULET_EINVAL;
    if (C) *C = b.C;
    if (H) *H = b.H;
    if (W) *W = b.W;
    if (elem_bytes) *elem_bytes = b.elem;
    if (ws_offset) *ws_offset = plan.offset[static_cast<size_t>(buf)];
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_run_model(const gpulet_model_desc *m, int batch, gpulet_partition *p,
                                          const void *in, void *out, void *workspace,
                                          size_t workspace_bytes, float *latency_ms) {
    if (!live(p)) return GPULET_EINVAL;
    Plan plan;
    gpulet_status st = build_plan(m, batch, plan);
    if (st != GPULET_OK) return st;
    st = check_run_args(plan, in, out, workspace, workspace_bytes);
    if (st != GPULET_OK) return st;
    const Bound bd{&plan, in, out, static_cast<char *>(workspace)};
    if (latency_ms) {
        EventPair ev;
        GPULET_HIP(ev.create());
        GPULET_HIP(timed_batch(bd, p, batch, ev, latency_ms));
        return GPULET_OK;
    }
    GPULET_HIP(enqueue(bd, p));
    p->batches_run.fetch_add(1);
    p->images_run.fetch_add(static_cast<uint64_t>(batch));
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_profile_model(const gpulet_model_desc *m, int batch,
                                              gpulet_partition *p, const void *in, void *out,
                                              void *workspace, size_t workspace_bytes, int warmup,
                                              int iters, int sync_each, float *latency_ms,
                                              float *total_ms) {
    if (!live(p) || iters < 1 || warmup < 0 || sync_each < 0 || sync_each > 2) return GPULET_EINVAL;
    if (sync_each == 2 ? !total_ms : !latency_ms) return GPULET_EINVAL;
    Plan plan;
    gpulet_status st = build_plan(m, batch, plan);
    if (st != GPULET_OK) return st;
    st = check_run_args(plan, in, out, workspace, workspace_bytes);
    if (st != GPULET_OK) return st;
    const Bound bd{&plan, in, out, static_cast<char *>(workspace)};

    for (int i = 0; i < warmup; ++i) {
        GPULET_HIP(enqueue(bd, p));
        p->batches_run.fetch_add(1);
        p->images_run.fetch_add(static_cast<uint64_t>(batch));
    }
    GPULET_HIP(hipStreamSynchronize(p->stream));

    if (sync_each == 2) {
        // one event pair around all batches
        EventPair e;
        GPULET_HIP(e.create());
        GPULET_HIP(hipEventRecord(e.a, p->stream));
        for (int i = 0; i < iters; ++i) {
            GPULET_HIP(enqueue(bd, p));
            p->batches_run.fetch_add(1);
            p->images_run.fetch_add(static_cast<uint64_t>(batch));
        }
        GPULET_HIP(hipEventRecord(e.b, p->stream));
        GPULET_HIP(hipEventSynchronize(e.b));
        GPULET_HIP(hipEventElapsedTime(total_ms, e.a, e.b));
        if (latency_ms)
            for (int i = 0; i < iters; ++i) latency_ms[i] = *total_ms / static_cast<float>(iters);
        return GPULET_OK;
    }
    std::vector<EventPair> ev(static_cast<size_t>(iters));
    for (EventPair &e : ev) GPULET_HIP(e.create());
    for (int i = 0; i < iters; ++i) {
        EventPair &e = ev[static_cast<size_t>(i)];
        GPULET_HIP(hipEventRecord(e.a, p->stream));
        GPULET_HIP(enqueue(bd, p));
        GPULET_HIP(hipEventRecord(e.b, p->stream));
        p->batches_run.fetch_add(1);
        p->images_run.fetch_add(static_cast<uint64_t>(batch));
        if (sync_each) GPULET_HIP(hipEventSynchronize(e.b));
    }
    GPULET_HIP(hipStreamSynchronize(p->stream));
    for (int i = 0; i < iters; ++i)
        GPULET_HIP(hipEventElapsedTime(&latency_ms[i], ev[static_cast<size_t>(i)].a, ev[static_cast<size_t>(i)].b));
    if (total_ms) GPULET_HIP(hipEventElapsedTime(total_ms, ev.front().a, ev.back().b));
    return GPULET_OK;
}

// A captured forward pass (one batch) bound to a gpu-let.
struct gpulet_graph {
    gpulet_partition *part;
    int batch;
    hipGraph_t graph;
    hipGraphExec_t exec;
};

namespace {

std::mutex g_graph_mu;
std::vector<gpulet_graph *> g_graphs;

bool graph_live(gpulet_graph *g) {
    if (!g) return false;
    std::lock_guard<std::mutex> lk(g_graph_mu);
    return std::find(g_graphs.begin(), g_graphs.end(), g) != g_graphs.end();
}

hipError_t timed_replay(gpulet_graph *g, EventPair &ev, float *ms) {
    gpulet_partition *p = g->part;
    hipError_t e = hipEventRecord(ev.a, p->stream);
    if (e == hipSuccess) e = hipGraphLaunch(g->exec, p->stream);
    if (e == hipSuccess) e = hipEventRecord(ev.b, p->stream);
    if (e == hipSuccess) e = hipEventSynchronize(ev.b);
    if (e == hipSuccess) e = hipEventElapsedTime(ms, ev.a, ev.b);
    if (e == hipSuccess) {
        p->batches_run.fetch_add(1);
        p->images_run.fetch_add(static_cast<uint64_t>(g->batch));
    }
    return e;
}

}  // namespace

extern "C" gpulet_status gpulet_model_graph_create(const gpulet_model_desc *m, int batch,
                                                   gpulet_partition *p, const void *in, void *out_buf,
                                                   void *workspace, size_t workspace_bytes,
                                                   gpulet_graph **out) {
    if (!out || !live(p)) return GPULET_EINVAL;
    Plan plan;
    gpulet_status st = build_plan(m, batch, plan);
    if (st != GPULET_OK) return st;
    st = check_run_args(plan, in, out_buf, workspace, workspace_bytes);
    if (st != GPULET_OK) return st;
    const Bound bd{&plan, in, out_buf, static_cast<char *>(workspace)};
    GPULET_HIP(hipStreamSynchronize(p->stream));
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    GPULET_HIP(hipStreamBeginCapture(p->stream, hipStreamCaptureModeThreadLocal));
    hipError_t e = enqueue(bd, p);
    hipError_t e2 = hipStreamEndCapture(p->stream, &graph);  // always end the capture
    if (e == hipSuccess) e = e2;
    if (e == hipSuccess) e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    if (e != hipSuccess) {
        if (graph) (void)hipGraphDestroy(graph);
        return hip_fail(e);
    }
    gpulet_graph *g = new gpulet_graph{p, batch, graph, exec};
    {
        std::lock_guard<std::mutex> lk(g_graph_mu);
        g_graphs.push_back(g);
    }
    *out = g;
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_model_graph_launch(gpulet_graph *g, float *latency_ms) {
    if (!graph_live(g) || !live(g->part)) return GPULET_EINVAL;
    if (latency_ms) {
        EventPair ev;
        GPULET_HIP(ev.create());
        GPULET_HIP(timed_replay(g, ev, latency_ms));
        return GPULET_OK;
    }
    GPULET_HIP(hipGraphLaunch(g->exec, g->part->stream));
    g->part->batches_run.fetch_add(1);
    g->part->images_run.fetch_add(static_cast<uint64_t>(g->batch));
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_model_graph_profile(gpulet_graph *g, int warmup, int iters,
                                                    float *latency_ms, float *total_ms) {
    if (!graph_live(g) || !live(g->part) || !latency_ms || iters < 1 || warmup < 0) return GPULET_EINVAL;
    EventPair ev;
    GPULET_HIP(ev.create());
    float ms = 0.f;
    for (int i = 0; i < warmup; ++i) GPULET_HIP(timed_replay(g, ev, &ms));
    const auto t0 = std::chrono::steady_clock::now();
    for (int i = 0; i < iters; ++i) GPULET_HIP(timed_replay(g, ev, &latency_ms[i]));
    if (total_ms)
        *total_ms = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - t0).count();
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_model_graph_destroy(gpulet_graph *g) {
    if (!g) return GPULET_EINVAL;
    {
        std::lock_guard<std::mutex> lk(g_graph_mu);
        auto it = std::find(g_graphs.begin(), g_graphs.end(), g);
        if (it == g_graphs.end()) return GPULET_EINVAL;
        g_graphs.erase(it);
    }
    hipError_t e = live(g->part) ? hipStreamSynchronize(g->part->stream) : hipSuccess;
    (void)hipGraphExecDestroy(g->exec);
    (void)hipGraphDestroy(g->graph);
    delete g;
    if (e != hipSuccess) return hip_fail(e);
    return GPULET_OK;
}

namespace {

struct CorunSide {
    const Plan *plan;
    Bound bd;
    gpulet_partition *p;
    int batch, warmup, cap;
    float *lat;
    int n = 0;
    gpulet_status status = GPULET_OK;
    int hip_error = 0;
};

// `done` / `other_done`: a side raises its flag when it leaves the window.  The batch a side is
// running when its neighbour leaves ran partly alone, so it is not reported (it still counts as a
// batch run on the gpu-let), and the side stops there: both sides' samples are co-run samples only.
void corun_thread(CorunSide *s, std::atomic<int> *ready, double window_ms, std::atomic<int> *done,
                  const std::atomic<int> *other_done) {
    auto fail = [&](hipError_t e) {
        s->status = GPULET_EHIP;
        s->hip_error = static_cast<int>(e);
    };
    hipError_t e = hipSetDevice(s->p->device);
    EventPair ev;
    if (e == hipSuccess) e = ev.create();
    for (int i = 0; i < s->warmup && e == hipSuccess; ++i) {
        float ms;
        e = timed_batch(s->bd, s->p, s->batch, ev, &ms);
    }
    // Both sides start their timed window together; a side that failed still
    // checks in so the other never waits forever.
    ready->fetch_add(1);
    while (ready->load() < 2) std::this_thread::yield();
    if (e != hipSuccess) {
        fail(e);
        done->store(1);
        return;
    }
    const auto t0 = std::chrono::steady_clock::now();
    for (;;) {
        float ms = 0.f;
        e = timed_batch(s->bd, s->p, s->batch, ev, &ms);
        if (e != hipSuccess) {
            fail(e);
            break;
        }
        if (other_done->load()) break;      // the neighbour left while this batch ran: not a co-run sample
        if (s->n < s->cap) s->lat[s->n] = ms;
        ++s->n;
        const double el = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
        if (el >= window_ms) break;
    }
    done->store(1);
}

}  // namespace

extern "C" gpulet_status gpulet_profile_corun(
    const gpulet_model_desc *ma, int batch_a, gpulet_partition *pa, const void *in_a, void *out_a,
    void *ws_a, size_t ws_a_bytes, const gpulet_model_desc *mb, int batch_b, gpulet_partition *pb,
    const void *in_b, void *out_b, void *ws_b, size_t ws_b_bytes, int warmup, double window_ms,
    float *lat_a, int cap_a, int *n_a, float *lat_b, int cap_b, int *n_b) {
    if (!live(pa) || !live(pb) || pa == pb || pa->device != pb->device) return GPULET_EINVAL;
    if (!lat_a || !lat_b || !n_a || !n_b || cap_a < 1 || cap_b < 1 || warmup < 0 || !(window_ms > 0.0))
        return GPULET_EINVAL;
    Plan plan_a, plan_b;
    gpulet_status st = build_plan(ma, batch_a, plan_a);
    if (st != GPULET_OK) return st;
    st = build_plan(mb, batch_b, plan_b);
    if (st != GPULET_OK) return st;
    st = check_run_args(plan_a, in_a, out_a, ws_a, ws_a_bytes);
    if (st != GPULET_OK) return st;
    st = check_run_args(plan_b, in_b, out_b, ws_b, ws_b_bytes);
    if (st != GPULET_OK) return st;

    CorunSide sa{&plan_a, Bound{&plan_a, in_a, out_a, static_cast<char *>(ws_a)}, pa, batch_a, warmup, cap_a, lat_a};
    CorunSide sb{&plan_b, Bound{&plan_b, in_b, out_b, static_cast<char *>(ws_b)}, pb, batch_b, warmup, cap_b, lat_b};
    std::atomic<int> ready{0}, done_a{0}, done_b{0};
    std::thread ta(corun_thread, &sa, &ready, window_ms, &done_a, &done_b);
    std::thread tb(corun_thread, &sb, &ready, window_ms, &done_b, &done_a);
    ta.join();
    tb.join();
    *n_a = std::min(sa.n, cap_a);
    *n_b = std::min(sb.n, cap_b);
    if (sa.status != GPULET_OK) return hip_fail(static_cast<hipError_t>(sa.hip_error));
    if (sb.status != GPULET_OK) return hip_fail(static_cast<hipError_t>(sb.hip_error));
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_latency_stats(const float *latency_ms, int n, double *mean,
                                              double *p50, double *p99) {
    if (!latency_ms || n < 1) return GPULET_EINVAL;
    std::vector<double> v(latency_ms, latency_ms + n);
    std::sort(v.begin(), v.end());
    double sum = 0.0;
    for (double d : v) sum += d;
    auto rank = [&](double pct) {
        int r = static_cast<int>(std::ceil(pct / 100.0 * n));
        r = std::max(1, std::min(n, r));
        return v[static_cast<size_t>(r - 1)];
    };
    if (mean) *mean = sum / n;
    if (p50) *p50 = rank(50.0);
    if (p99) *p99 = rank(99.0);
    return GPULET_OK;
}
