// gpu-let manager: creates CU-masked streams and keeps the per-device and
// per-partition bookkeeping (paper Sec. 2.3; Sec. 1: at most two gpu-lets per
// GPU; Sec. 4.3 Split: sizes p and 100-p).
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "gpulet_internal.h"

namespace gpulet {

static thread_local int t_last_hip_error = 0;

gpulet_status hip_fail(hipError_t e) {
    t_last_hip_error = static_cast<int>(e);
    return GPULET_EHIP;
}

namespace {

std::mutex g_mu;
std::vector<gpulet_partition *> g_live;  // every live gpu-let, all devices

// Dies per device.  The KFD topology states it (num_xcc); fall back to 8, the
// MI355X layout, when the count divides the CUs, else to one die.
int xcd_count(int n_cu_total) {
    if (const char *env = std::getenv("GPULET_N_XCD")) {
        const int v = std::atoi(env);
        if (v > 0 && n_cu_total % v == 0) return v;
    }
    for (int node = 0; node < 64; ++node) {
        char path[128];
        std::snprintf(path, sizeof path, "/sys/class/kfd/kfd/topology/nodes/%d/properties", node);
        FILE *f = std::fopen(path, "r");
        if (!f) continue;
        char key[64];
        unsigned long long val;
        int simd = 0, xcc = 0;
        while (std::fscanf(f, "%63s %llu", key, &val) == 2) {
            if (!std::strcmp(key, "simd_count")) simd = static_cast<int>(val);
            if (!std::strcmp(key, "num_xcc")) xcc = static_cast<int>(val);
        }
        std::fclose(f);
        if (simd > 0 && xcc > 0 && n_cu_total % xcc == 0) return xcc;
    }
    return n_cu_total % 8 == 0 ? 8 : 1;
}

}  // namespace

bool live(const gpulet_partition *p) {
    if (!p) return false;
    std::lock_guard<std::mutex> lk(g_mu);
    for (const gpulet_partition *q : g_live)
        if (q == p) return true;
    return false;
}

LaunchCtx partition_ctx(const gpulet_partition *p) {
    LaunchCtx c;
    c.n_cu = p->n_cu;
    c.scratch = static_cast<float *>(p->scratch);
    c.scratch_bytes = p->scratch_bytes;
    c.counters = p->counters;
    c.n_counters = p->n_counters;
    return c;
}

LaunchCtx stream_ctx(hipStream_t stream) {
    {
        std::lock_guard<std::mutex> lk(g_mu);
        for (const gpulet_partition *p : g_live)
            if (p->stream == stream) return partition_ctx(p);
    }
    LaunchCtx c;
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
        c.n_cu = n;
    return c;
}

}  // namespace gpulet

using namespace gpulet;

extern "C" int gpulet_last_hip_error(void) { return t_last_hip_error; }

extern "C" gpulet_status gpulet_partition_create(int device, int pct, int which,
                                                 gpulet_partition **out) {
    if (!out) return GPULET_EINVAL;
    if (pct < 1 || pct > 100 || which < 0 || which > 1 || device < 0) return GPULET_EINVAL;
    int n_dev = 0;
    GPULET_HIP(hipGetDeviceCount(&n_dev));
    if (device >= n_dev) return GPULET_EINVAL;
    int n_cu_total = 0;
    GPULET_HIP(hipDeviceGetAttribute(&n_cu_total, hipDeviceAttributeMultiprocessorCount, device));
    if (n_cu_total < 1 || n_cu_total > 32 * kMaxMaskWords) return GPULET_EINVAL;

    uint32_t words[kMaxMaskWords] = {0};
    int n_words = 0, n_cu = 0;
    gpulet_status st = gpulet_mask_for_pct(n_cu_total, xcd_count(n_cu_total), pct, which, words,
                                           kMaxMaskWords, &n_words, &n_cu);
    if (st != GPULET_OK) return st;

    std::lock_guard<std::mutex> lk(g_mu);
    int live_here = 0, pct_here = 0;
    for (const gpulet_partition *q : g_live) {
        if (q->device != device) continue;
        ++live_here;
        pct_here += q->pct;
        if (q->which == which) return GPULET_EOVERSUB;
    }
    if (live_here >= 2 || pct_here + pct > 100) return GPULET_EOVERSUB;

    int prev = 0;
    GPULET_HIP(hipGetDevice(&prev));
    GPULET_HIP(hipSetDevice(device));
    hipStream_t stream = nullptr;
    hipStream_t extra[kMaxLanes] = {nullptr};
    hipError_t e = hipExtStreamCreateWithCUMask(&stream, static_cast<uint32_t>(n_words), words);
    // The second lane is switched off (gpulet_set_model_lanes), so its stream is not created.
    constexpr bool kCreateLanes = false;
    for (int l = 1; l < kMaxLanes && e == hipSuccess && kCreateLanes; ++l)
        e = hipExtStreamCreateWithCUMask(&extra[l], static_cast<uint32_t>(n_words), words);
    // Split-K scratch of the gpu-let: partial tiles and zeroed arrival counters.
    constexpr size_t kScratchBytes = 64u << 20;
    constexpr int kCounters = 4096;
    void *scratch = nullptr;
    unsigned *counters = nullptr;
    if (e == hipSuccess) e = hipMalloc(&scratch, kScratchBytes);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&counters), kCounters * sizeof(unsigned));
    if (e == hipSuccess) e = hipMemset(counters, 0, kCounters * sizeof(unsigned));
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        if (scratch) (void)hipFree(scratch);
        if (counters) (void)hipFree(counters);
        if (stream) (void)hipStreamDestroy(stream);
        for (int l = 1; l < kMaxLanes; ++l)
            if (extra[l]) (void)hipStreamDestroy(extra[l]);
        (void)hipSetDevice(prev);
        return hip_fail(e);
    }
    (void)hipSetDevice(prev);

    gpulet_partition *p = new gpulet_partition();
    p->device = device;
    p->pct = pct;
    p->which = which;
    p->n_cu = n_cu;
    p->n_cu_total = n_cu_total;
    p->n_words = n_words;
    std::memcpy(p->mask, words, sizeof words);
    p->stream = stream;
    p->lane[0] = stream;
    for (int l = 1; l < kMaxLanes; ++l) p->lane[l] = extra[l];
    p->scratch = scratch;
    p->scratch_bytes = kScratchBytes;
    p->counters = counters;
    p->n_counters = kCounters;
    p->batches_run.store(0);
    p->images_run.store(0);
    p->kernels_enqueued.store(0);
    g_live.push_back(p);
    *out = p;
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_partition_destroy(gpulet_partition *p) {
    if (!p) return GPULET_EINVAL;
    hipStream_t stream;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        size_t i = 0;
        for (; i < g_live.size(); ++i)
            if (g_live[i] == p) break;
        if (i == g_live.size()) return GPULET_EINVAL;  // unknown or already destroyed
        g_live.erase(g_live.begin() + static_cast<long>(i));
        stream = p->stream;
    }
    hipError_t e1 = hipStreamSynchronize(stream);
    for (int l = 1; l < kMaxLanes; ++l) {
        if (!p->lane[l]) continue;
        hipError_t el = hipStreamSynchronize(p->lane[l]);
        if (e1 == hipSuccess) e1 = el;
        (void)hipStreamDestroy(p->lane[l]);
    }
    for (hipEvent_t ev : p->events) (void)hipEventDestroy(ev);
    hipError_t e2 = hipStreamDestroy(stream);
    (void)hipFree(p->scratch);
    (void)hipFree(p->counters);
    delete p;
    if (e1 != hipSuccess) return hip_fail(e1);
    if (e2 != hipSuccess) return hip_fail(e2);
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_partition_info(const gpulet_partition *p, int *device, int *pct,
                                               int *which, int *n_cu, int *n_cu_total,
                                               uint32_t mask_words[8], int *n_words,
                                               void **hip_stream) {
    if (!live(p)) return GPULET_EINVAL;
    if (device) *device = p->device;
    if (pct) *pct = p->pct;
    if (which) *which = p->which;
    if (n_cu) *n_cu = p->n_cu;
    if (n_cu_total) *n_cu_total = p->n_cu_total;
    if (mask_words) std::memcpy(mask_words, p->mask, sizeof p->mask);
    if (n_words) *n_words = p->n_words;
    if (hip_stream) *hip_stream = static_cast<void *>(p->stream);
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_partition_query_mask(const gpulet_partition *p,
                                                     uint32_t mask_words[8], int *n_words) {
    if (!live(p) || !mask_words) return GPULET_EINVAL;
    std::memset(mask_words, 0, sizeof(uint32_t) * kMaxMaskWords);
    GPULET_HIP(hipExtStreamGetCUMask(p->stream, static_cast<uint32_t>(p->n_words), mask_words));
    if (n_words) *n_words = p->n_words;
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_partition_counters(const gpulet_partition *p, uint64_t *batches_run,
                                                   uint64_t *images_run) {
    if (!live(p)) return GPULET_EINVAL;
    if (batches_run) *batches_run = p->batches_run.load();
    if (images_run) *images_run = p->images_run.load();
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_partition_kernel_launches(const gpulet_partition *p, uint64_t *launches) {
    if (!live(p) || !launches) return GPULET_EINVAL;
    *launches = p->kernels_enqueued.load();
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_partition_sync(gpulet_partition *p) {
    if (!live(p)) return GPULET_EINVAL;
    GPULET_HIP(hipStreamSynchronize(p->stream));
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_partition_probe_ex(gpulet_partition *p, uint32_t *out, int n_blocks,
                                                   int via_graph) {
    if (!live(p) || !out || n_blocks < 1) return GPULET_EINVAL;
    if (!via_graph) {
        GPULET_HIP(launch_probe(out, n_blocks, p->stream));
        GPULET_HIP(hipStreamSynchronize(p->stream));
        return GPULET_OK;
    }
    GPULET_HIP(hipStreamSynchronize(p->stream));
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    GPULET_HIP(hipStreamBeginCapture(p->stream, hipStreamCaptureModeThreadLocal));
    hipError_t e = launch_probe(out, n_blocks, p->stream);
    hipError_t e2 = hipStreamEndCapture(p->stream, &graph);
    if (e == hipSuccess) e = e2;
    if (e == hipSuccess) e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    if (e == hipSuccess) e = hipGraphLaunch(exec, p->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(p->stream);
    if (exec) (void)hipGraphExecDestroy(exec);
    if (graph) (void)hipGraphDestroy(graph);
    if (e != hipSuccess) return hip_fail(e);
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_partition_mfma_rate(gpulet_partition *p, int dense, int waves_per_cu, int iters,
                                                    int launches, float *avg_ms, double *tflops) {
    if (!live(p) || !avg_ms || !tflops || iters < 1 || launches < 1) return GPULET_EINVAL;
    if (waves_per_cu != 4 && waves_per_cu != 8) return GPULET_EINVAL;
    const int blocks = p->n_cu;
    if (static_cast<size_t>(blocks) * waves_per_cu * 64 * sizeof(float) > p->scratch_bytes) return GPULET_ENOMEM;
    float *out = static_cast<float *>(p->scratch);
    GPULET_HIP(launch_mfma_rate(out, blocks, waves_per_cu, iters, dense, p->stream));  // warm-up
    hipEvent_t e0 = nullptr, e1 = nullptr;
    GPULET_HIP(hipEventCreate(&e0));
    hipError_t e = hipEventCreate(&e1);
    if (e != hipSuccess) {
        (void)hipEventDestroy(e0);
        return hip_fail(e);
    }
    e = hipEventRecord(e0, p->stream);
    for (int i = 0; i < launches && e == hipSuccess; ++i)
        e = launch_mfma_rate(out, blocks, waves_per_cu, iters, dense, p->stream);
    if (e == hipSuccess) e = hipEventRecord(e1, p->stream);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return hip_fail(e);
    *avg_ms = ms / static_cast<float>(launches);
    const double flop = 2.0 * 32 * 32 * 16 * 64.0 * iters * waves_per_cu * blocks;  // per launch
    *tflops = flop / (static_cast<double>(*avg_ms) * 1e-3) * 1e-12;
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_partition_probe(gpulet_partition *p, uint32_t *out, int n_blocks) {
    return gpulet_partition_probe_ex(p, out, n_blocks, 0);
}
