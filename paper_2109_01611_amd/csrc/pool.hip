// Pooling layers of the forward pass served on a gpu-let (paper Sec. 5; models
// of Table 4), NHWC bf16.  These are bandwidth-bound: each thread owns 8
// consecutive channels of one output pixel (one 16-byte load per tap, adjacent
// lanes adjacent in memory).  Global average pooling splits the H x W plane
// over 8 lane groups of a wavefront and combines the partial fp32 sums with a
// wavefront shuffle reduction.
#include <hip/hip_runtime.h>

#include "gpulet_internal.h"
#include "pool_device.h"

namespace gpulet {
namespace {

__device__ __forceinline__ float bf16_bits_to_f32(unsigned short h) {
    return __uint_as_float(static_cast<unsigned>(h) << 16);
}

__device__ __forceinline__ unsigned short f32_to_bf16_bits(float f) {
    const __bf16 h = static_cast<__bf16>(f);
    return *reinterpret_cast<const unsigned short *>(&h);
}

__device__ __forceinline__ void unpack8(const uint4 &v, float f[8]) {
    const unsigned u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(u[i] << 16);
        f[2 * i + 1] = __uint_as_float(u[i] & 0xFFFF0000u);
    }
}

__device__ __forceinline__ uint4 pack8(const float f[8]) {
    unsigned u[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        u[i] = static_cast<unsigned>(f32_to_bf16_bits(f[2 * i])) |
               (static_cast<unsigned>(f32_to_bf16_bits(f[2 * i + 1])) << 16);
    return make_uint4(u[0], u[1], u[2], u[3]);
}

// Window pooling, 8 channels per thread.  AVG = false: max over in-image taps.
// AVG = true: sum of in-image taps / (k*k).  K > 0 fixes the window size at
// compile time: all K*K loads are then issued before the first one is used
// (taps outside the image load a clamped address and are masked afterwards), so
// a thread pays the memory latency once instead of once per tap; these kernels
// are small enough for that latency to be most of their run time.  K = 0 is the
// general loop.
template <bool AVG, int K>
__global__ __launch_bounds__(256) void pool_window_vec8(const PoolParams p) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= p.total) return;
    const int cv = p.C >> 3;
    const int c8 = idx % cv;
    int t = idx / cv;
    const int q = t % p.Q;
    t /= p.Q;
    const int pp = t % p.P;
    const int n = t / p.P;
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = AVG ? 0.f : -INFINITY;
    const int h0 = pp * p.stride - p.pad, w0 = q * p.stride - p.pad;
    if (K > 0) {
        uint4 v[K > 0 ? K * K : 1];
        bool ok[K > 0 ? K * K : 1];
#pragma unroll
        for (int r = 0; r < K; ++r)
#pragma unroll
            for (int s = 0; s < K; ++s) {
                const int h = h0 + r, w = w0 + s;
                ok[r * K + s] = ((unsigned)h < (unsigned)p.H) & ((unsigned)w < (unsigned)p.W);
                const int hc = min(max(h, 0), p.H - 1), wc = min(max(w, 0), p.W - 1);
                v[r * K + s] = *reinterpret_cast<const uint4 *>(p.x + (((n * p.H + hc) * p.W + wc) * p.C + c8 * 8));
            }
#pragma unroll
        for (int j = 0; j < K * K; ++j) {
            float f[8];
            unpack8(v[j], f);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (AVG)
                    acc[i] += ok[j] ? f[i] : 0.f;
                else
                    acc[i] = ok[j] ? fmaxf(acc[i], f[i]) : acc[i];
            }
        }
    } else {
        for (int r = 0; r < p.k; ++r) {
            const int h = h0 + r;
            if ((unsigned)h >= (unsigned)p.H) continue;
            for (int s = 0; s < p.k; ++s) {
                const int w = w0 + s;
                if ((unsigned)w >= (unsigned)p.W) continue;
                const uint4 v = *reinterpret_cast<const uint4 *>(p.x + (((n * p.H + h) * p.W + w) * p.C + c8 * 8));
                float f[8];
                unpack8(v, f);
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] = AVG ? acc[i] + f[i] : fmaxf(acc[i], f[i]);
            }
        }
    }
    if (AVG) {
        const float inv = 1.f / static_cast<float>(p.k * p.k);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] *= inv;
    }
    *reinterpret_cast<uint4 *>(p.y + (((n * p.P + pp) * p.Q + q) * p.C + c8 * 8)) = pack8(acc);
}

// Max pooling with a K x K window, K fixed at compile time (every max pool of the served
// models is 2x2 or 3x3): 8 channels of one output pixel per thread as above, but nothing is
// converted to fp32 and nothing is masked.  Window coordinates are clamped to the image, which
// only repeats taps that are in the window anyway (pad < K and floor-mode extents guarantee
// that a window starts and ends inside the image once clamped), so padding never wins; all K*K
// loads are issued first; the maximum is taken on order-preserving integer keys; the index
// arithmetic is multiply-shift.  About half the instructions of the general kernel.
template <int K>
__global__ __launch_bounds__(256) void pool_max_vec8(const PoolParams p) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= p.total) return;
    pool_max_item<K>(p, idx);
}

// Window pooling for channel counts that are not multiples of 8: one element per thread.
template <bool AVG>
__global__ __launch_bounds__(256) void pool_window_scalar(const PoolParams p) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= p.total) return;
    const int c = idx % p.C;
    int t = idx / p.C;
    const int q = t % p.Q;
    t /= p.Q;
    const int pp = t % p.P;
    const int n = t / p.P;
    float acc = AVG ? 0.f : -INFINITY;
    const int h0 = pp * p.stride - p.pad, w0 = q * p.stride - p.pad;
    const unsigned short *xs = reinterpret_cast<const unsigned short *>(p.x);
    for (int r = 0; r < p.k; ++r) {
        const int h = h0 + r;
        if ((unsigned)h >= (unsigned)p.H) continue;
        for (int s = 0; s < p.k; ++s) {
            const int w = w0 + s;
            if ((unsigned)w >= (unsigned)p.W) continue;
            const float f = bf16_bits_to_f32(xs[((n * p.H + h) * p.W + w) * p.C + c]);
            acc = AVG ? acc + f : fmaxf(acc, f);
        }
    }
    if (AVG) acc *= 1.f / static_cast<float>(p.k * p.k);
    reinterpret_cast<unsigned short *>(p.y)[idx] = f32_to_bf16_bits(acc);
}

// Global average pooling.  A wavefront covers 8 groups of 8 channels; its 64
// lanes are 8 plane slices x 8 channel groups.  Lane (slice, group) sums pixels
// slice, slice + 8, ... of its channels in fp32, then the 8 slices are folded
// with three xor-shuffles and slice 0 stores.  `total` counts wavefronts.
__global__ __launch_bounds__(256) void pool_global_avg_vec8(const PoolParams p) {
    const int wave = (blockIdx.x * 256 + threadIdx.x) >> 6;
    if (wave >= p.total) return;  // whole wavefronts leave together
    const int lane = threadIdx.x & 63;
    const int group = lane & 7, slice = lane >> 3;
    const int cv = p.C >> 3;
    const int groups_per_img = (cv + 7) >> 3;  // wavefronts per image
    const int n = wave / groups_per_img;
    const int c8 = (wave - n * groups_per_img) * 8 + group;
    const int hw = p.H * p.W;
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    if (c8 < cv) {
        for (int i = slice; i < hw; i += 8) {
            const uint4 v = *reinterpret_cast<const uint4 *>(p.x + ((n * hw + i) * p.C + c8 * 8));
            float f[8];
            unpack8(v, f);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] += f[j];
        }
    }
#pragma unroll
    for (int off = 8; off < 64; off <<= 1)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] += __shfl_xor(acc[j], off, 64);
    if (slice == 0 && c8 < cv) {
        const float inv = 1.f / static_cast<float>(hw);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] *= inv;
        *reinterpret_cast<uint4 *>(p.y + (n * p.C + c8 * 8)) = pack8(acc);
    }
}

// Global average pooling, any channel count: one wavefront per (image, channel),
// lanes stride the plane, full wavefront reduction.  `total` counts wavefronts.
__global__ __launch_bounds__(256) void pool_global_avg_scalar(const PoolParams p) {
    const int wave = (blockIdx.x * 256 + threadIdx.x) >> 6;
    if (wave >= p.total) return;
    const int lane = threadIdx.x & 63;
    const int n = wave / p.C, c = wave - n * p.C;
    const int hw = p.H * p.W;
    const unsigned short *xs = reinterpret_cast<const unsigned short *>(p.x);
    float acc = 0.f;
    for (int i = lane; i < hw; i += 64) acc += bf16_bits_to_f32(xs[(n * hw + i) * p.C + c]);
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) reinterpret_cast<unsigned short *>(p.y)[wave] = f32_to_bf16_bits(acc / static_cast<float>(hw));
}

}  // namespace

gpulet_status check_pool(int N, int C, int H, int W, int mode, int k, int stride, int pad, int *P,
                         int *Q) {
    if (N < 1 || C < 1 || H < 1 || W < 1) return GPULET_EINVAL;
    if (mode != GPULET_POOL_MAX && mode != GPULET_POOL_AVG && mode != GPULET_POOL_GLOBAL_AVG)
        return GPULET_EINVAL;
    if (1LL * N * H * W * C >= (1LL << 31)) return GPULET_EINVAL;
    if (mode == GPULET_POOL_GLOBAL_AVG) {
        *P = 1;
        *Q = 1;
        return GPULET_OK;
    }
    if (k < 1 || stride < 1 || pad < 0 || pad >= k) return GPULET_EINVAL;
    *P = out_extent(H, k, stride, pad);
    *Q = out_extent(W, k, stride, pad);
    if (*P < 1 || *Q < 1) return GPULET_EINVAL;
    return GPULET_OK;
}

hipError_t launch_pool(const void *x, void *y, int N, int C, int H, int W, int P, int Q, int mode,
                       int k, int stride, int pad, hipStream_t stream) {
    PoolParams p;
    p.x = static_cast<const __bf16 *>(x);
    p.y = static_cast<__bf16 *>(y);
    p.N = N; p.C = C; p.H = H; p.W = W; p.P = P; p.Q = Q; p.k = k; p.stride = stride; p.pad = pad;
    const bool vec = (C % 8 == 0) && (reinterpret_cast<uintptr_t>(x) % 16 == 0) &&
                     (reinterpret_cast<uintptr_t>(y) % 16 == 0);
    if (mode == GPULET_POOL_GLOBAL_AVG) {
        p.total = vec ? N * ((C / 8 + 7) / 8) : N * C;  // wavefronts
        const unsigned blocks = static_cast<unsigned>((p.total + 3) / 4);
        if (vec)
            hipLaunchKernelGGL(pool_global_avg_vec8, dim3(blocks), dim3(256), 0, stream, p);
        else
            hipLaunchKernelGGL(pool_global_avg_scalar, dim3(blocks), dim3(256), 0, stream, p);
        return hipGetLastError();
    }
    p.total = vec ? N * P * Q * (C / 8) : N * P * Q * C;
    const unsigned blocks = static_cast<unsigned>((p.total + 255) / 256);
    const bool avg = mode == GPULET_POOL_AVG;
    if (vec && !avg && (k == 2 || k == 3)) {
        p.d_cv = make_fastdiv(C / 8);
        p.d_q = make_fastdiv(Q);
        p.d_p = make_fastdiv(P);
        if (k == 3)
            hipLaunchKernelGGL(pool_max_vec8<3>, dim3(blocks), dim3(256), 0, stream, p);
        else
            hipLaunchKernelGGL(pool_max_vec8<2>, dim3(blocks), dim3(256), 0, stream, p);
    } else if (vec) {
#define GPULET_POOL_LAUNCH(K) \
    do { \
        if (avg) hipLaunchKernelGGL((pool_window_vec8<true, K>), dim3(blocks), dim3(256), 0, stream, p); \
        else hipLaunchKernelGGL((pool_window_vec8<false, K>), dim3(blocks), dim3(256), 0, stream, p); \
    } while (0)
        if (k == 3) GPULET_POOL_LAUNCH(3);
        else if (k == 2) GPULET_POOL_LAUNCH(2);
        else GPULET_POOL_LAUNCH(0);
#undef GPULET_POOL_LAUNCH
    } else {
        if (avg)
            hipLaunchKernelGGL(pool_window_scalar<true>, dim3(blocks), dim3(256), 0, stream, p);
        else
            hipLaunchKernelGGL(pool_window_scalar<false>, dim3(blocks), dim3(256), 0, stream, p);
    }
    return hipGetLastError();
}

}  // namespace gpulet
