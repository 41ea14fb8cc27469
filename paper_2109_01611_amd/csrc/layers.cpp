// Single-layer entry points of the C ABI: argument checks, then a launch on
// the caller's stream (paper Sec. 5: the executor runs the model's layers on
// its gpu-let).
#include <cstdint>

#include "gpulet_internal.h"

using namespace gpulet;

namespace {

gpulet_status make_conv_args(ConvArgs &a, const void *x, const void *w, const float *b, void *y,
                             int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                             int relu, const void *residual, int y_ch_stride, int y_ch_offset) {
    a.x = x; a.w = w; a.b = b; a.y = y; a.residual = residual;
    a.N = N; a.C = C; a.H = H; a.W = W; a.K = K; a.R = R; a.S = S;
    a.stride = stride; a.pad = pad; a.relu = relu ? 1 : 0;
    a.y_ch_stride = y_ch_stride == 0 ? K : y_ch_stride;
    a.y_ch_offset = y_ch_offset;
    if (stride < 1 || R < 1 || S < 1 || pad < 0 || H < 1 || W < 1) return GPULET_EINVAL;
    a.P = out_extent(H, R, stride, pad);
    a.Q = out_extent(W, S, stride, pad);
    return check_conv(a);
}

}  // namespace

extern "C" gpulet_status gpulet_conv2d_fwd_ex(const void *x, const void *w, const float *b, void *y,
                                              int N, int C, int H, int W, int K, int R, int S,
                                              int stride, int pad, int relu, const void *residual,
                                              int y_ch_stride, int y_ch_offset, void *stream) {
    ConvArgs a;
    gpulet_status st = make_conv_args(a, x, w, b, y, N, C, H, W, K, R, S, stride, pad, relu, residual,
                                      y_ch_stride, y_ch_offset);
    if (st != GPULET_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    GPULET_HIP(launch_conv(a, stream_ctx(s), s));
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_conv2d_fwd_slices(const void *x, const void *w, const float *b, void *y, int N,
                                                  int C, int H, int W, int K, int R, int S, int stride,
                                                  int pad, int relu, const void *residual, int x_ch_stride,
                                                  int x_ch_offset, int y_ch_stride, int y_ch_offset,
                                                  void *stream) {
    ConvArgs a;
    a.x_ch_stride = x_ch_stride;
    a.x_ch_offset = x_ch_offset;
    gpulet_status st = make_conv_args(a, x, w, b, y, N, C, H, W, K, R, S, stride, pad, relu, residual,
                                      y_ch_stride, y_ch_offset);
    if (st != GPULET_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    GPULET_HIP(launch_conv(a, stream_ctx(s), s));
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_conv1x1_fwd_two_outputs(const void *x, const void *w, const float *b, void *y,
                                                        void *y2, int N, int C, int H, int W, int K, int k2,
                                                        int stride, int relu, int x_ch_stride, int x_ch_offset,
                                                        int y_ch_stride, int y_ch_offset, int y2_ch_stride,
                                                        int y2_ch_offset, void *stream) {
    if (!y2 || k2 < 1 || k2 >= K) return GPULET_EINVAL;
    ConvArgs a;
    a.x_ch_stride = x_ch_stride;
    a.x_ch_offset = x_ch_offset;
    a.y2 = y2;
    a.k2 = k2;
    a.y2_ch_stride = y2_ch_stride == 0 ? K - k2 : y2_ch_stride;
    a.y2_ch_offset = y2_ch_offset;
    gpulet_status st = make_conv_args(a, x, w, b, y, N, C, H, W, K, 1, 1, stride, 0, relu, nullptr,
                                      y_ch_stride == 0 ? k2 : y_ch_stride, y_ch_offset);
    if (st != GPULET_OK) return st;
    const int ldx = x_ch_stride ? x_ch_stride : C;
    if (C % 8 != 0 || ldx % 8 != 0 || x_ch_offset % 8 != 0 || reinterpret_cast<uintptr_t>(x) % 16 != 0 ||
        reinterpret_cast<uintptr_t>(w) % 16 != 0)
        return GPULET_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    GPULET_HIP(launch_conv(a, stream_ctx(s), s));
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_conv2d_group_fwd(const gpulet_conv_desc *layers, int n, void *stream) {
    if (!layers || n < 1 || n > kMaxGroup) return GPULET_EINVAL;
    ConvArgs a[kMaxGroup];
    struct Range { uintptr_t lo, hi; };
    Range xr[kMaxGroup], rr[kMaxGroup], yr[kMaxGroup];
    for (int j = 0; j < n; ++j) {
        const gpulet_conv_desc &d = layers[j];
        a[j].x_ch_stride = d.x_ch_stride;
        a[j].x_ch_offset = d.x_ch_offset;
        gpulet_status st = make_conv_args(a[j], d.x, d.w, d.b, d.y, d.N, d.C, d.H, d.W, d.K, d.R, d.S, d.stride,
                                          d.pad, d.relu, d.residual, d.y_ch_stride, d.y_ch_offset);
        if (st != GPULET_OK) return st;
        const uintptr_t ldx = static_cast<uintptr_t>(d.x_ch_stride ? d.x_ch_stride : d.C);
        const uintptr_t px = static_cast<uintptr_t>(d.N) * d.H * d.W, py = static_cast<uintptr_t>(d.N) * a[j].P * a[j].Q;
        xr[j] = {reinterpret_cast<uintptr_t>(d.x), reinterpret_cast<uintptr_t>(d.x) + 2 * px * ldx};
        rr[j] = {reinterpret_cast<uintptr_t>(d.residual),
                 d.residual ? reinterpret_cast<uintptr_t>(d.residual) + 2 * py * d.K : 0};
        yr[j] = {reinterpret_cast<uintptr_t>(d.y), reinterpret_cast<uintptr_t>(d.y) + 2 * py * a[j].y_ch_stride};
    }
    auto meet = [](const Range &p, const Range &q) { return p.lo < q.hi && q.lo < p.hi; };
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) {
            if (i == j) continue;
            if (meet(yr[i], xr[j]) || (rr[j].hi && meet(yr[i], rr[j]))) return GPULET_EINVAL;
            if (i < j && meet(yr[i], yr[j])) {
                // only as disjoint channel slices of one tensor
                const bool slices = a[i].y == a[j].y && a[i].y_ch_stride == a[j].y_ch_stride && a[i].P == a[j].P &&
                                    a[i].Q == a[j].Q && a[i].N == a[j].N &&
                                    (a[i].y_ch_offset + a[i].K <= a[j].y_ch_offset ||
                                     a[j].y_ch_offset + a[j].K <= a[i].y_ch_offset);
                if (!slices) return GPULET_EINVAL;
            }
        }
    hipStream_t s = static_cast<hipStream_t>(stream);
    GPULET_HIP(launch_conv_group(a, n, stream_ctx(s), s));
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_conv1x1_maxpool3_fwd(const void *x, const void *w, const float *b, void *y,
                                                     void *y2, void *pool_y, int N, int C, int H, int W, int K,
                                                     int k2, int relu, int y_ch_stride, int y_ch_offset,
                                                     int y2_ch_stride, int y2_ch_offset, void *stream) {
    if (!pool_y || reinterpret_cast<uintptr_t>(pool_y) % 16 != 0) return GPULET_EINVAL;
    if (y2 && (k2 < 1 || k2 >= K)) return GPULET_EINVAL;
    ConvArgs a;
    a.pool_y = pool_y;
    const int k1 = y2 ? k2 : K;
    if (y2) {
        a.y2 = y2;
        a.k2 = k2;
        a.y2_ch_stride = y2_ch_stride == 0 ? K - k2 : y2_ch_stride;
        a.y2_ch_offset = y2_ch_offset;
    }
    gpulet_status st = make_conv_args(a, x, w, b, y, N, C, H, W, K, 1, 1, 1, 0, relu, nullptr,
                                      y_ch_stride == 0 ? k1 : y_ch_stride, y_ch_offset);
    if (st != GPULET_OK) return st;
    if (reinterpret_cast<uintptr_t>(x) % 16 != 0 || reinterpret_cast<uintptr_t>(w) % 16 != 0) return GPULET_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    GPULET_HIP(launch_conv(a, stream_ctx(s), s));
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_maxpool3_conv1x1_fwd(const void *x, const void *w, const float *b, void *y, int N,
                                                     int C, int H, int W, int K, int relu, int y_ch_stride,
                                                     int y_ch_offset, void *stream) {
    ConvArgs a;
    a.pre_pool = 3;
    gpulet_status st = make_conv_args(a, x, w, b, y, N, C, H, W, K, 1, 1, 1, 0, relu, nullptr, y_ch_stride,
                                      y_ch_offset);
    if (st != GPULET_OK) return st;
    if (reinterpret_cast<uintptr_t>(x) % 16 != 0 || reinterpret_cast<uintptr_t>(w) % 16 != 0) return GPULET_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    GPULET_HIP(launch_conv(a, stream_ctx(s), s));
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_conv3x3_maxpool2_fwd(const void *x, const void *w, const float *b, void *y, int N,
                                                     int C, int H, int W, int K, int y_ch_stride, int y_ch_offset,
                                                     void *stream) {
    ConvArgs a;
    a.post_pool2 = 2;
    gpulet_status st = make_conv_args(a, x, w, b, y, N, C, H, W, K, 3, 3, 1, 1, 1, nullptr, y_ch_stride, y_ch_offset);
    if (st != GPULET_OK) return st;
    // what the kernel with the pooled epilogue needs: whole 64-channel blocks, 16-byte stores
    if (C % 64 != 0 || K % 8 != 0 || a.y_ch_stride % 8 != 0 || a.y_ch_offset % 8 != 0 ||
        reinterpret_cast<uintptr_t>(x) % 16 != 0 || reinterpret_cast<uintptr_t>(w) % 16 != 0 ||
        reinterpret_cast<uintptr_t>(y) % 16 != 0 || reinterpret_cast<uintptr_t>(b) % 16 != 0)
        return GPULET_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    GPULET_HIP(launch_conv(a, stream_ctx(s), s));
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_set_conv_pool_fusion(int on) {
    if (on != 0 && on != 1) return GPULET_EINVAL;
    set_conv_pool_fusion(on);
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_conv2d_fwd(const void *x, const void *w, const float *b, void *y,
                                           int N, int C, int H, int W, int K, int R, int S,
                                           int stride, int pad, int relu, void *stream) {
    return gpulet_conv2d_fwd_ex(x, w, b, y, N, C, H, W, K, R, S, stride, pad, relu, nullptr, 0, 0,
                                stream);
}

extern "C" gpulet_status gpulet_conv2d_timeline(const void *x, const void *w, const float *b, void *y, int N, int C,
                                                int H, int W, int K, int R, int S, int stride, int pad, int relu,
                                                void *stream, int warmup, int64_t *stamps, int *workgroups) {
    if (!stamps || !workgroups || warmup < 0) return GPULET_EINVAL;
    ConvArgs a;
    gpulet_status st = make_conv_args(a, x, w, b, y, N, C, H, W, K, R, S, stride, pad, relu, nullptr, 0, 0);
    if (st != GPULET_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const LaunchCtx ctx = stream_ctx(s);
    constexpr size_t kBytes = 8 * 8 * sizeof(int64_t);
    void *dev = nullptr;
    GPULET_HIP(hipMalloc(&dev, kBytes));
    hipError_t e = hipMemsetAsync(dev, 0, kBytes, s);
    for (int i = 0; i < warmup && e == hipSuccess; ++i) e = launch_conv(a, ctx, s);
    a.stamps = dev;
    if (e == hipSuccess) e = launch_conv(a, ctx, s);
    if (e == hipSuccess) e = hipMemcpyAsync(stamps, dev, kBytes, hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    (void)hipFree(dev);
    if (e != hipSuccess) return hip_fail(e);
    int n = 0;
    while (n < 8 && stamps[n * 8] != 0) ++n;
    *workgroups = n;
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_set_conv_tile(int tile) {
    if (tile < -1 || tile >= GPULET_CONV_TILES) return GPULET_EINVAL;
    set_conv_tile(tile);
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_set_conv_split_k(int max_split) {
    if (max_split < 1 || max_split > 8) return GPULET_EINVAL;
    set_conv_split_k(max_split);
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_depthwise_conv2d_fwd(const void *x, const void *w, const float *b, void *y,
                                                     int N, int C, int H, int W, int R, int S, int stride,
                                                     int pad, int relu, void *stream) {
    if (!x || !w || !y) return GPULET_EINVAL;
    int P = 0, Q = 0;
    gpulet_status st = check_dwconv(N, C, H, W, R, S, stride, pad, &P, &Q);
    if (st != GPULET_OK) return st;
    GPULET_HIP(launch_dwconv(x, w, b, y, N, C, H, W, R, S, stride, pad, relu ? 1 : 0, P, Q,
                             static_cast<hipStream_t>(stream)));
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_pool(const void *x, void *y, int N, int C, int H, int W, int mode,
                                     int k, int stride, int pad, void *stream) {
    if (!x || !y) return GPULET_EINVAL;
    int P = 0, Q = 0;
    gpulet_status st = check_pool(N, C, H, W, mode, k, stride, pad, &P, &Q);
    if (st != GPULET_OK) return st;
    GPULET_HIP(launch_pool(x, y, N, C, H, W, P, Q, mode, k, stride, pad, static_cast<hipStream_t>(stream)));
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_fc(const void *x, const void *w, const float *b, void *y, int N,
                                   int In, int Out, int relu, int out_fp32, void *stream) {
    if (!x || !w || !y) return GPULET_EINVAL;
    gpulet_status st = check_fc(N, In, Out);
    if (st != GPULET_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    GPULET_HIP(launch_fc(x, w, b, y, N, In, Out, relu ? 1 : 0, out_fp32 ? 1 : 0, stream_ctx(s), s));
    return GPULET_OK;
}

extern "C" gpulet_status gpulet_fc_static_scratch(const void *x, const void *w, const float *b, void *y, int N,
                                                  int In, int Out, int relu, int out_fp32, void *stream) {
    if (!x || !w || !y) return GPULET_EINVAL;
    gpulet_status st = check_fc(N, In, Out);
    if (st != GPULET_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    bool too_large = false;
    GPULET_HIP(launch_fc_static(x, w, b, y, N, In, Out, relu ? 1 : 0, out_fp32 ? 1 : 0, stream_ctx(s).n_cu, s,
                                &too_large));
    return too_large ? GPULET_ENOMEM : GPULET_OK;
}

extern "C" gpulet_status gpulet_time_conv2d(const void *x, const void *w, const float *b, void *y,
                                            int N, int C, int H, int W, int K, int R, int S,
                                            int stride, int pad, int relu, const void *residual,
                                            int y_ch_stride, int y_ch_offset, void *stream,
                                            int warmup, int iters, float *avg_ms) {
    if (!avg_ms || iters < 1 || warmup < 0) return GPULET_EINVAL;
    ConvArgs a;
    gpulet_status st = make_conv_args(a, x, w, b, y, N, C, H, W, K, R, S, stride, pad, relu, residual,
                                      y_ch_stride, y_ch_offset);
    if (st != GPULET_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const LaunchCtx ctx = stream_ctx(s);
    for (int i = 0; i < warmup; ++i) GPULET_HIP(launch_conv(a, ctx, s));
    hipEvent_t e0 = nullptr, e1 = nullptr;
    GPULET_HIP(hipEventCreate(&e0));
    hipError_t e = hipEventCreate(&e1);
    if (e != hipSuccess) {
        (void)hipEventDestroy(e0);
        return hip_fail(e);
    }
    e = hipEventRecord(e0, s);
    for (int i = 0; i < iters && e == hipSuccess; ++i) e = launch_conv(a, ctx, s);
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return hip_fail(e);
    *avg_ms = ms / static_cast<float>(iters);
    return GPULET_OK;
}
