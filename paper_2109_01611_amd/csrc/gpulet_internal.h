// Internal declarations shared by the translation units of libgpulet.so.
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
#include <cstddef>
#include <cstdint>
#include <vector>

#include "gpulet.h"

namespace gpulet {

// Records the failing hipError_t for gpulet_last_hip_error() and returns GPULET_EHIP.
gpulet_status hip_fail(hipError_t e);

#define GPULET_HIP(expr)                                   \
    do {                                                   \
        hipError_t e__ = (expr);                           \
        if (e__ != hipSuccess) return ::gpulet::hip_fail(e__); \
    } while (0)

constexpr int kMaxMaskWords = 8;
// Streams of one gpu-let, all with its CU mask.  Independent layers of a model (inception
// branches, a projection shortcut next to the main path, detection heads) may run on different
// lanes at once.  Two gpu-lets of two lanes fill the four hardware queues of a process.
constexpr int kMaxLanes = 2;

}  // namespace gpulet

// A live gpu-let (paper Sec. 2.3): a CU-masked stream plus its bookkeeping.
struct gpulet_partition {
    int device;
    int pct;
    int which;
    int n_cu;
    int n_cu_total;
    int n_words;
    uint32_t mask[gpulet::kMaxMaskWords];
    hipStream_t stream;     // lane 0: what callers see, where batches are ordered and timed
    hipStream_t lane[gpulet::kMaxLanes];  // lane[0] == stream
    std::vector<hipEvent_t> events;       // ordering events between lanes, grown on demand by the model runner
    void *scratch;          // device memory for split-K partial tiles, owned by the gpu-let
    size_t scratch_bytes;
    unsigned *counters;     // device arrival counters for split-K, zero between launches
    int n_counters;
    std::atomic<uint64_t> batches_run;
    std::atomic<uint64_t> images_run;
    std::atomic<uint64_t> kernels_enqueued;  // kernel launches of eager model runs (a launch group counts once)
};

namespace gpulet {

// True if p is a handle gpulet_partition_create returned and nobody destroyed yet
// (looked up in the registry, so a stale pointer is never dereferenced).
bool live(const gpulet_partition *p);

// Output extent of a window op; <= 0 means empty.
inline int out_extent(int in, int k, int stride, int pad) {
    const int span = in + 2 * pad - k;
    return span < 0 ? 0 : span / stride + 1;
}

// What a launch on a stream may use: the CU count tile selection keys on and, for
// a gpu-let's stream, the gpu-let's private split-K scratch (none otherwise, which
// switches split-K off).  Work on one stream is serial, so the scratch is never shared.
struct LaunchCtx {
    int n_cu = 256;
    float *scratch = nullptr;
    size_t scratch_bytes = 0;
    unsigned *counters = nullptr;
    int n_counters = 0;
};
LaunchCtx stream_ctx(hipStream_t stream);
LaunchCtx partition_ctx(const gpulet_partition *p);

// Kernel launchers (conv.hip, dwconv.hip, pool.hip, fc.hip).  Arguments are validated by the callers.
constexpr int kMaxGroup = 4;  // layers per launch group

struct ConvArgs {
    const void *x, *w;
    const float *b;
    void *y;
    const void *residual;
    int N, C, H, W, K, R, S, stride, pad, relu, P, Q, y_ch_stride, y_ch_offset;
    int pre_pool = 0;  // 3: a 3x3 / stride 1 / pad 1 max pool is applied to x first (1x1 filters only)
    // The layer reads channels [x_ch_offset, x_ch_offset + C) of pixels that hold x_ch_stride
    // channels (0: the pixels hold exactly C).
    int x_ch_stride = 0, x_ch_offset = 0;
    // Second destination (1x1 filters, no residual): when y2 is set, filters [k2, K) are stored to
    // channels [y2_ch_offset, y2_ch_offset + K - k2) of y2's pixels (y2_ch_stride channels each)
    // and only filters [0, k2) to y.
    void *y2 = nullptr;
    int k2 = 0, y2_ch_stride = 0, y2_ch_offset = 0;
    // Side job (1x1 filters, dense input, C % 8 == 0): when set, the launch also writes the
    // 3x3 / stride 1 / pad 1 max pool of x (N*H*W*C bf16) to pool_y.
    void *pool_y = nullptr;
    // 2: a 2x2 / stride 2 max pool follows and y receives only the pooled tensor (N, P/2, Q/2 pixels
    // of y_ch_stride channels); P and Q stay the layer's own output size.  Only layers for which
    // conv_pool2_fusable() holds.
    int post_pool2 = 0;
    // Measurement (gpulet_conv2d_timeline): device array of 8 x 8 int64 that the kernel's first
    // workgroups fill with wall-clock stamps, if the kernel that runs the layer records them.
    void *stamps = nullptr;
};
hipError_t launch_conv(const ConvArgs &a, const LaunchCtx &ctx, hipStream_t stream);
// Whether the layer followed by a 2x2 / stride 2 max pool should run as one launch on this
// stream: a kernel that can pool in its epilogue applies (3x3, stride 1, pad 1, ReLU, no residual,
// C a multiple of 64, even output size, aligned dense operands) and is the kernel the layer would
// run anyway (64 input channels, weights in registers) or at most a few percent slower on the
// layer alone (the tall tile, from 128 channels on).  `a.y` is the pooled destination.
bool conv_pool2_fusable(const ConvArgs &a, const LaunchCtx &ctx);
void set_conv_pool_fusion(int on);
// n independent layers (no member reads or overwrites what another writes), in one launch where
// the kernels allow it.
// *launches (if not null) receives the number of kernel launches made: 1 or n.
hipError_t launch_conv_group(const ConvArgs *a, int n, const LaunchCtx &ctx, hipStream_t stream,
                             int *launches = nullptr);
void set_conv_tile(int tile);
void set_conv_split_k(int max_split);
hipError_t launch_pool(const void *x, void *y, int N, int C, int H, int W, int P, int Q, int mode,
                       int k, int stride, int pad, hipStream_t stream);
hipError_t launch_fc(const void *x, const void *w, const float *b, void *y, int N, int In, int Out,
                     int relu, int out_fp32, const LaunchCtx &ctx, hipStream_t stream);
// The layer with its scratch in the library's static device array (no allocation anywhere);
// *too_large is set, and nothing launched, when the layer needs more than the array holds.
hipError_t launch_fc_static(const void *x, const void *w, const float *b, void *y, int N, int In, int Out,
                            int relu, int out_fp32, int n_cu, hipStream_t stream, bool *too_large);
hipError_t launch_dwconv(const void *x, const void *w, const float *b, void *y, int N, int C, int H, int W,
                         int R, int S, int stride, int pad, int relu, int P, int Q, hipStream_t stream);
hipError_t launch_probe(uint32_t *out, int n_blocks, hipStream_t stream);
// blocks x waves wavefronts of nothing but 32x32x16 bf16 matrix instructions, 64 * iters each; out: one float
// per thread.  dense: pseudo-random operands in (-1, 1) instead of zeros.
hipError_t launch_mfma_rate(float *out, int blocks, int waves, int iters, int dense, hipStream_t stream);

// Argument checks shared by the single-layer entry points and the model runner.
gpulet_status check_conv(const ConvArgs &a);
gpulet_status check_pool(int N, int C, int H, int W, int mode, int k, int stride, int pad, int *P,
                         int *Q);
gpulet_status check_fc(int N, int In, int Out);
gpulet_status check_dwconv(int N, int C, int H, int W, int R, int S, int stride, int pad, int *P, int *Q);

}  // namespace gpulet
