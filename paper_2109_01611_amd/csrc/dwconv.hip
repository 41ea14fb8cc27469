// Depthwise convolution of the forward pass served on a gpu-let (paper Sec. 5;
// the SSD-MobileNet of Table 4 is built from depthwise 3x3 + pointwise 1x1
// pairs), NHWC bf16, filter [R][S][C] bf16, fp32 accumulation, fused bias and
// ReLU, one rounding to bf16.
//
// One multiply-add per loaded input element: the layer is bound by memory
// traffic, not by arithmetic, so there is nothing for the matrix cores to do.
// Each thread owns 8 consecutive channels (one 16-byte load per tap, adjacent
// lanes adjacent in memory) of TQ horizontally adjacent output pixels, so the
// taps neighbouring pixels share are loaded once per thread and the filter
// once per TQ pixels; the remaining overlap between threads is served by the
// caches.  Algorithmic bytes: 2*(N*H*W*C + N*P*Q*C + R*S*C) + 4*C.
#include <hip/hip_runtime.h>

#include "device_util.h"
#include "gpulet_internal.h"

namespace gpulet {
namespace {

struct DwParams {
    const __bf16 *x, *w;
    const float *b;
    __bf16 *y;
    int N, C, H, W, R, S, stride, pad, relu, P, Q;
    int qt;     // thread columns per output row = ceil(Q / TQ)
    int total;  // work items
    FastDiv d_cv, d_qt, d_p;  // 3x3 kernel: divisions by C/8, qt and P
};

__device__ __forceinline__ void unpack8(const uint4 &v, float f[8]) {
    const unsigned u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(u[i] << 16);
        f[2 * i + 1] = __uint_as_float(u[i] & 0xFFFF0000u);
    }
}

__device__ __forceinline__ unsigned short bf16_bits(float f) {
    const __bf16 h = static_cast<__bf16>(f);
    return *reinterpret_cast<const unsigned short *>(&h);
}

template <int TQ>
__global__ __launch_bounds__(256) void dwconv_vec8(const DwParams p) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= p.total) return;
    const int cv = p.C >> 3;
    const int c8 = idx % cv;
    int t = idx / cv;
    const int qg = t % p.qt;
    t /= p.qt;
    const int pp = t % p.P;
    const int n = t / p.P;
    const int q0 = qg * TQ;

    float acc[TQ][8];
    float bias[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (p.b) {
        const float4 b0 = *reinterpret_cast<const float4 *>(p.b + c8 * 8);
        const float4 b1 = *reinterpret_cast<const float4 *>(p.b + c8 * 8 + 4);
        bias[0] = b0.x; bias[1] = b0.y; bias[2] = b0.z; bias[3] = b0.w;
        bias[4] = b1.x; bias[5] = b1.y; bias[6] = b1.z; bias[7] = b1.w;
    }
#pragma unroll
    for (int j = 0; j < TQ; ++j)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[j][i] = bias[i];

    const int h0 = pp * p.stride - p.pad;
    const int w_first = q0 * p.stride - p.pad;               // input column of tap 0 of the first pixel
    const int span = (TQ - 1) * p.stride + p.S;              // input columns the TQ pixels touch
    for (int r = 0; r < p.R; ++r) {
        const int h = h0 + r;
        if ((unsigned)h >= (unsigned)p.H) continue;
        const __bf16 *xrow = p.x + ((n * p.H + h) * p.W) * p.C + c8 * 8;
        const __bf16 *wrow = p.w + (r * p.S) * p.C + c8 * 8;
        for (int u = 0; u < span; ++u) {
            const int w = w_first + u;
            if ((unsigned)w >= (unsigned)p.W) continue;
            float xv[8];
            unpack8(*reinterpret_cast<const uint4 *>(xrow + w * p.C), xv);
            // input column u is tap s = u - j*stride of pixel j
#pragma unroll
            for (int j = 0; j < TQ; ++j) {
                const int s = u - j * p.stride;
                if (s < 0 || s >= p.S) continue;
                float wv[8];
                unpack8(*reinterpret_cast<const uint4 *>(wrow + s * p.C), wv);
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[j][i] = fmaf(xv[i], wv[i], acc[j][i]);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < TQ; ++j) {
        const int q = q0 + j;
        if (q >= p.Q) break;
        unsigned o[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float a = acc[j][2 * i], b = acc[j][2 * i + 1];
            if (p.relu) {
                a = a > 0.f ? a : 0.f;
                b = b > 0.f ? b : 0.f;
            }
            o[i] = static_cast<unsigned>(bf16_bits(a)) | (static_cast<unsigned>(bf16_bits(b)) << 16);
        }
        *reinterpret_cast<uint4 *>(p.y + (((n * p.P + pp) * p.Q + q) * p.C + c8 * 8)) =
            make_uint4(o[0], o[1], o[2], o[3]);
    }
}

// 3x3 filters (every depthwise layer of MobileNet): the generic kernel above walks rows and
// columns in loops with tests, so each of its 18 loads waits for the previous one's use, and a
// layer of 24 MB took 20 us.  Here the taps are unrolled at compile time and every input load
// (buffer loads: an offset pushed out of range returns zero, so padding needs no branch) and
// every filter load is issued before the first multiply-add.  Same work split (8 channels x TQ
// adjacent pixels per thread) and the same summation order, so the bits are those of the kernel
// above.
typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;

template <int STRIDE, int TQ>
__global__ __launch_bounds__(256) void dwconv3x3_vec8(const DwParams p, const unsigned x_bytes) {
    constexpr int SPAN = (TQ - 1) * STRIDE + 3;  // input columns the TQ pixels touch
    constexpr unsigned OOB = 0x80000000u;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= p.total) return;
    const int cv = p.C >> 3;
    int t = fdiv(idx, p.d_cv);
    const int c8 = idx - t * cv;
    const int t1 = fdiv(t, p.d_qt);
    const int qg = t - t1 * p.qt;
    const int n = fdiv(t1, p.d_p);
    const int pp = t1 - n * p.P;
    const int q0 = qg * TQ;
    const int h0 = pp * STRIDE - p.pad, w_first = q0 * STRIDE - p.pad;

    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<__bf16 *>(p.x), 0, x_bytes, 0x00020000);
    u32x4_t xr[3][SPAN];
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int h = h0 + r;
        const bool h_ok = static_cast<unsigned>(h) < static_cast<unsigned>(p.H);
        const int row = ((n * p.H + h) * p.W + w_first) * p.C + c8 * 8;
#pragma unroll
        for (int u = 0; u < SPAN; ++u) {
            const bool ok = h_ok && static_cast<unsigned>(w_first + u) < static_cast<unsigned>(p.W);
            xr[r][u] = __builtin_amdgcn_raw_buffer_load_b128(rx, ok ? static_cast<unsigned>((row + u * p.C) * 2) : OOB, 0, 0);
        }
    }
    uint4 wr[3][3];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int sx = 0; sx < 3; ++sx) wr[r][sx] = *reinterpret_cast<const uint4 *>(p.w + (r * 3 + sx) * p.C + c8 * 8);

    float acc[TQ][8];
    {
        float bias[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (p.b) {
            const float4 b0 = *reinterpret_cast<const float4 *>(p.b + c8 * 8);
            const float4 b1 = *reinterpret_cast<const float4 *>(p.b + c8 * 8 + 4);
            bias[0] = b0.x; bias[1] = b0.y; bias[2] = b0.z; bias[3] = b0.w;
            bias[4] = b1.x; bias[5] = b1.y; bias[6] = b1.z; bias[7] = b1.w;
        }
#pragma unroll
        for (int j = 0; j < TQ; ++j)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[j][i] = bias[i];
    }
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        float wv[3][8];
#pragma unroll
        for (int sx = 0; sx < 3; ++sx) unpack8(wr[r][sx], wv[sx]);
#pragma unroll
        for (int u = 0; u < SPAN; ++u) {
            float xv[8];
            unpack8(make_uint4(xr[r][u][0], xr[r][u][1], xr[r][u][2], xr[r][u][3]), xv);
#pragma unroll
            for (int j = 0; j < TQ; ++j) {
                const int sx = u - j * STRIDE;  // input column u is tap sx of pixel j
                if (sx < 0 || sx >= 3) continue;
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[j][i] = fmaf(xv[i], wv[sx][i], acc[j][i]);
            }
        }
    }
    const unsigned limit = relu_limit(p.relu);
#pragma unroll
    for (int j = 0; j < TQ; ++j) {
        const int q = q0 + j;
        if (q >= p.Q) break;
        unsigned o[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = relu_or_pass(pack_bf16(acc[j][2 * i], acc[j][2 * i + 1]), limit);
        *reinterpret_cast<uint4 *>(p.y + (((n * p.P + pp) * p.Q + q) * p.C + c8 * 8)) =
            make_uint4(o[0], o[1], o[2], o[3]);
    }
}

// Any channel count or alignment: one thread per output element.
__global__ __launch_bounds__(256) void dwconv_scalar(const DwParams p) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= p.total) return;
    const int c = idx % p.C;
    int t = idx / p.C;
    const int q = t % p.Q;
    t /= p.Q;
    const int pp = t % p.P;
    const int n = t / p.P;
    float acc = p.b ? p.b[c] : 0.f;
    for (int r = 0; r < p.R; ++r) {
        const int h = pp * p.stride - p.pad + r;
        if ((unsigned)h >= (unsigned)p.H) continue;
        for (int s = 0; s < p.S; ++s) {
            const int w = q * p.stride - p.pad + s;
            if ((unsigned)w >= (unsigned)p.W) continue;
            acc = fmaf(static_cast<float>(p.x[((n * p.H + h) * p.W + w) * p.C + c]),
                       static_cast<float>(p.w[(r * p.S + s) * p.C + c]), acc);
        }
    }
    if (p.relu) acc = acc > 0.f ? acc : 0.f;
    p.y[idx] = static_cast<__bf16>(acc);
}

}  // namespace

gpulet_status check_dwconv(int N, int C, int H, int W, int R, int S, int stride, int pad, int *P, int *Q) {
    if (N < 1 || C < 1 || H < 1 || W < 1 || R < 1 || S < 1 || stride < 1 || pad < 0) return GPULET_EINVAL;
    *P = out_extent(H, R, stride, pad);
    *Q = out_extent(W, S, stride, pad);
    if (*P < 1 || *Q < 1) return GPULET_EINVAL;
    const long long lim = 1LL << 30;
    if (1LL * N * H * W * C >= lim || 1LL * N * *P * *Q * C >= lim || 1LL * R * S * C >= lim) return GPULET_EINVAL;
    return GPULET_OK;
}

hipError_t launch_dwconv(const void *x, const void *w, const float *b, void *y, int N, int C, int H, int W,
                         int R, int S, int stride, int pad, int relu, int P, int Q, hipStream_t stream) {
    DwParams p;
    p.x = static_cast<const __bf16 *>(x);
    p.w = static_cast<const __bf16 *>(w);
    p.b = b;
    p.y = static_cast<__bf16 *>(y);
    p.N = N; p.C = C; p.H = H; p.W = W; p.R = R; p.S = S; p.stride = stride; p.pad = pad; p.relu = relu;
    p.P = P; p.Q = Q;
    const bool vec = (C % 8 == 0) && reinterpret_cast<uintptr_t>(x) % 16 == 0 &&
                     reinterpret_cast<uintptr_t>(w) % 16 == 0 && reinterpret_cast<uintptr_t>(y) % 16 == 0 &&
                     reinterpret_cast<uintptr_t>(b) % 16 == 0;
    if (vec && R == 3 && S == 3 && (stride == 1 || stride == 2)) {
        const unsigned x_bytes = static_cast<unsigned>(2LL * N * H * W * C);
        p.d_cv = make_fastdiv(C / 8);
        p.d_p = make_fastdiv(P);
        p.d_qt = make_fastdiv((Q + (stride == 1 ? 4 : 2) - 1) / (stride == 1 ? 4 : 2));
        if (stride == 1) {
            constexpr int TQ = 4;
            p.qt = (Q + TQ - 1) / TQ;
            p.total = N * P * p.qt * (C / 8);
            hipLaunchKernelGGL((dwconv3x3_vec8<1, TQ>), dim3((p.total + 255) / 256), dim3(256), 0, stream, p, x_bytes);
        } else {
            constexpr int TQ = 2;
            p.qt = (Q + TQ - 1) / TQ;
            p.total = N * P * p.qt * (C / 8);
            hipLaunchKernelGGL((dwconv3x3_vec8<2, TQ>), dim3((p.total + 255) / 256), dim3(256), 0, stream, p, x_bytes);
        }
    } else if (vec) {
        constexpr int TQ = 4;
        p.qt = (Q + TQ - 1) / TQ;
        p.total = N * P * p.qt * (C / 8);
        hipLaunchKernelGGL(dwconv_vec8<TQ>, dim3((p.total + 255) / 256), dim3(256), 0, stream, p);
    } else {
        p.qt = Q;
        p.total = N * P * Q * C;
        hipLaunchKernelGGL(dwconv_scalar, dim3((p.total + 255) / 256), dim3(256), 0, stream, p);
    }
    return hipGetLastError();
}

}  // namespace gpulet
