// Fully connected layer of the forward pass served on a gpu-let (paper Sec. 5;
// classifier heads of the models in Table 4) on gfx950 matrix cores.
//
// At serving batch sizes (1-32, Fig. 3) this GEMM has as many rows as the
// batch, so it is bound by streaming the [Out][In] weights from HBM once.
// A workgroup owns 16 outputs and up to 32 batch rows; its wavefronts (4, or 16
// for long rows) each stream a contiguous share of the In range straight from global memory into
// v_mfma_f32_16x16x32_bf16 operands (no LDS staging: every weight is used
// once), then the partial accumulators are summed through LDS and the
// first wavefront adds bias, applies ReLU and stores bf16 or fp32.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>

#include "gpulet_internal.h"

namespace gpulet {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

struct FcParams {
    const __bf16 *x, *w;
    const float *b;
    void *y;
    int N, In, Out, relu, out_fp32;
};

constexpr int UNROLL = 4;  // depth steps of 32 in flight per wavefront

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4 &v) {
    return *reinterpret_cast<const bf16x8 *>(&v);
}

// Loads 8 consecutive elements starting at row_ptr[k]; zero where out of range.
template <bool VEC>
__device__ __forceinline__ uint4 load_chunk(const __bf16 *row_ptr, int k, int In, bool row_ok) {
    if (VEC) {
        if (row_ok && k < In) return *reinterpret_cast<const uint4 *>(row_ptr + k);
        return make_uint4(0u, 0u, 0u, 0u);
    }
    unsigned short e[8];
    const unsigned short *s = reinterpret_cast<const unsigned short *>(row_ptr);
#pragma unroll
    for (int i = 0; i < 8; ++i) e[i] = (row_ok && k + i < In) ? s[k + i] : (unsigned short)0;
    return make_uint4(e[0] | ((unsigned)e[1] << 16), e[2] | ((unsigned)e[3] << 16),
                      e[4] | ((unsigned)e[5] << 16), e[6] | ((unsigned)e[7] << 16));
}

// NB = batch tiles of 16 rows handled per workgroup (1 or 2); NW = wavefronts
// that split the In range (4, or 16 for long rows so that enough loads are in
// flight per CU to keep HBM busy).
template <int NB, int NW, bool VEC>
__global__ __launch_bounds__(NW * 64) void fc_kernel(const FcParams p) {
    __shared__ float red[NW - 1][NB][64][4];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int o0 = blockIdx.x * 16;
    const int n0 = blockIdx.y * (16 * NB);
    const int sub = lane & 15;   // operand row (batch row for x, output for w)
    const int kq = lane >> 4;    // which 8 of the 32 depth elements of a step

    const int o = o0 + sub;
    const bool o_ok = o < p.Out;
    const __bf16 *wrow = p.w + static_cast<size_t>(o_ok ? o : 0) * p.In;
    const __bf16 *xrow[NB];
    bool n_ok[NB];
#pragma unroll
    for (int t = 0; t < NB; ++t) {
        const int n = n0 + t * 16 + sub;
        n_ok[t] = n < p.N;
        xrow[t] = p.x + static_cast<size_t>(n_ok[t] ? n : 0) * p.In;
    }

    const int steps = (p.In + 31) / 32;
    const int per_wave = (steps + NW - 1) / NW;
    const int s_begin = wave * per_wave;
    const int s_end = min(steps, s_begin + per_wave);

    f32x4 acc[NB];
#pragma unroll
    for (int t = 0; t < NB; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int s = s_begin; s < s_end; s += UNROLL) {
        uint4 rw[UNROLL], rx[NB][UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int k = (s + u) * 32 + kq * 8;
            const bool live = s + u < s_end;
            rw[u] = load_chunk<VEC>(wrow, k, p.In, o_ok && live);
#pragma unroll
            for (int t = 0; t < NB; ++t) rx[t][u] = load_chunk<VEC>(xrow[t], k, p.In, n_ok[t] && live);
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
#pragma unroll
            for (int t = 0; t < NB; ++t)
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(rx[t][u]), as_bf16x8(rw[u]),
                                                                 acc[t], 0, 0, 0);
    }

    if (wave > 0) {
#pragma unroll
        for (int t = 0; t < NB; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) red[wave - 1][t][lane][v] = acc[t][v];
    }
    __syncthreads();
    if (wave != 0) return;

    // Accumulator register v of a lane holds batch row 4*(lane/16) + v, output lane%16.
    const float bias = (p.b && o_ok) ? p.b[o] : 0.f;
#pragma unroll
    for (int t = 0; t < NB; ++t) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float val = acc[t][v];
#pragma unroll
            for (int w = 0; w < NW - 1; ++w) val += red[w][t][lane][v];
            const int n = n0 + t * 16 + 4 * kq + v;
            if (!o_ok || n >= p.N) continue;
            val += bias;
            if (p.relu) val = val > 0.f ? val : 0.f;
            const size_t idx = static_cast<size_t>(n) * p.Out + o;
            if (p.out_fp32)
                static_cast<float *>(p.y)[idx] = val;
            else
                static_cast<__bf16 *>(p.y)[idx] = static_cast<__bf16>(val);
        }
    }
}

// Long rows (In >= 8192: the first classifier layer of VGG-16, 25088 -> 4096).  With 16
// outputs per workgroup every one of the Out/16 workgroups reads the whole activation matrix
// from L2, which at batch 32 is twice the bytes of the weights themselves and held the layer at
// 2.3 TB/s of weight traffic.  Here a workgroup owns 64 outputs (four 16-wide blocks share
// every activation fragment) and one of `ksplit` contiguous ranges of the depth, so the grid
// still fills the chip; its 16 wavefronts split that range and are summed through LDS as above.
// The `ksplit` partial tiles of an output group meet in device scratch: each workgroup stores
// its tile with device-scope stores, waits for them, and counts itself in with one atomic; the
// last to arrive (nobody waits) adds the tiles in split order and finishes.  The sum order is
// fixed, so results are reproducible, and the same kernel serves every batch size, so an image's
// result does not depend on its batch.
template <int NB, bool VEC>
__global__ __launch_bounds__(1024) void fc_split_kernel(const FcParams p, float *part, unsigned *cnt, const int ksplit,
                                                        const int steps_per_split) {
    constexpr int NW = 16, OB = 4;  // wavefronts; 16-output blocks per workgroup
    __shared__ float red[NW - 1][NB * OB][64][4];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int og = blockIdx.x, ks = blockIdx.y;
    const int o0 = og * (16 * OB);
    const int sub = lane & 15, kq = lane >> 4;

    const __bf16 *wrow[OB];
    bool o_ok[OB];
#pragma unroll
    for (int j = 0; j < OB; ++j) {
        const int o = o0 + j * 16 + sub;
        o_ok[j] = o < p.Out;
        wrow[j] = p.w + static_cast<size_t>(o_ok[j] ? o : 0) * p.In;
    }
    const __bf16 *xrow[NB];
    bool n_ok[NB];
#pragma unroll
    for (int t = 0; t < NB; ++t) {
        const int n = t * 16 + sub;
        n_ok[t] = n < p.N;
        xrow[t] = p.x + static_cast<size_t>(n_ok[t] ? n : 0) * p.In;
    }

    const int steps = (p.In + 31) / 32;
    const int r_begin = ks * steps_per_split, r_end = min(steps, r_begin + steps_per_split);
    const int per_wave = (max(r_end - r_begin, 0) + NW - 1) / NW;
    const int s_begin = r_begin + wave * per_wave;
    const int s_end = min(r_end, s_begin + per_wave);

    f32x4 acc[NB][OB];
#pragma unroll
    for (int t = 0; t < NB; ++t)
#pragma unroll
        for (int j = 0; j < OB; ++j) acc[t][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    constexpr int U = NB == 1 ? 4 : 2;  // depth steps of 32 in flight per wavefront: (4 + NB) loads each
    for (int s = s_begin; s < s_end; s += U) {
        uint4 rw[OB][U], rx[NB][U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k = (s + u) * 32 + kq * 8;
            const bool live = s + u < s_end;
#pragma unroll
            for (int j = 0; j < OB; ++j) rw[j][u] = load_chunk<VEC>(wrow[j], k, p.In, o_ok[j] && live);
#pragma unroll
            for (int t = 0; t < NB; ++t) rx[t][u] = load_chunk<VEC>(xrow[t], k, p.In, n_ok[t] && live);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < NB; ++t)
#pragma unroll
                for (int j = 0; j < OB; ++j)
                    acc[t][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(rx[t][u]), as_bf16x8(rw[j][u]),
                                                                         acc[t][j], 0, 0, 0);
    }

    if (wave > 0) {
#pragma unroll
        for (int t = 0; t < NB; ++t)
#pragma unroll
            for (int j = 0; j < OB; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) red[wave - 1][t * OB + j][lane][v] = acc[t][j][v];
    }
    __syncthreads();
    if (wave != 0) return;
#pragma unroll
    for (int t = 0; t < NB; ++t)
#pragma unroll
        for (int j = 0; j < OB; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float val = acc[t][j][v];
#pragma unroll
                for (int w = 0; w < NW - 1; ++w) val += red[w][t * OB + j][lane][v];
                acc[t][j][v] = val;
            }

    if (ksplit > 1) {
        constexpr int DEVICE_SCOPE = 16;  // cache policy sc1: device scope, bypasses the die-local caches
        constexpr int TILE_BYTES = NB * OB * 64 * 16;
        const __amdgpu_buffer_rsrc_t rp =
            __builtin_amdgcn_make_buffer_rsrc(part, 0, static_cast<int>(gridDim.x) * ksplit * TILE_BYTES, 0x00020000);
        const int mine = (og * ksplit + ks) * TILE_BYTES;
#pragma unroll
        for (int t = 0; t < NB; ++t)
#pragma unroll
            for (int j = 0; j < OB; ++j) {
                typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;
                const u32x4_t bits = {__float_as_uint(acc[t][j][0]), __float_as_uint(acc[t][j][1]),
                                      __float_as_uint(acc[t][j][2]), __float_as_uint(acc[t][j][3])};
                __builtin_amdgcn_raw_buffer_store_b128(bits, rp, mine + ((t * OB + j) * 64 + lane) * 16, 0, DEVICE_SCOPE);
            }
        __builtin_amdgcn_s_waitcnt(0);  // the wavefront's partial tile has reached memory
        unsigned arrived = 0;
        if (lane == 0) {
            arrived = __hip_atomic_fetch_add(&cnt[og], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (arrived == static_cast<unsigned>(ksplit - 1))  // ready for the next launch
                __hip_atomic_store(&cnt[og], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        arrived = __builtin_amdgcn_readfirstlane(arrived);
        if (arrived != static_cast<unsigned>(ksplit - 1)) return;
#pragma unroll
        for (int t = 0; t < NB; ++t)
#pragma unroll
            for (int j = 0; j < OB; ++j) acc[t][j] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int q = 0; q < ksplit; ++q) {
            typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;
            u32x4_t raw[NB * OB];
#pragma unroll
            for (int i = 0; i < NB * OB; ++i)  // all loads of one partial tile in flight together
                raw[i] = __builtin_amdgcn_raw_buffer_load_b128(rp, (og * ksplit + q) * TILE_BYTES + (i * 64 + lane) * 16, 0,
                                                               DEVICE_SCOPE);
#pragma unroll
            for (int t = 0; t < NB; ++t)
#pragma unroll
                for (int j = 0; j < OB; ++j)
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[t][j][v] += __uint_as_float(raw[t * OB + j][v]);
        }
    }

    // Accumulator register v of a lane holds batch row 4*(lane/16) + v, output lane%16.
#pragma unroll
    for (int j = 0; j < OB; ++j) {
        const int o = o0 + j * 16 + sub;
        if (!o_ok[j]) continue;
        const float bias = p.b ? p.b[o] : 0.f;
#pragma unroll
        for (int t = 0; t < NB; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int n = t * 16 + 4 * kq + v;
                if (n >= p.N) continue;
                float val = acc[t][j][v] + bias;
                if (p.relu) val = val > 0.f ? val : 0.f;
                const size_t idx = static_cast<size_t>(n) * p.Out + o;
                if (p.out_fp32)
                    static_cast<float *>(p.y)[idx] = val;
                else
                    static_cast<__bf16 *>(p.y)[idx] = static_cast<__bf16>(val);
            }
    }
}

}  // namespace

gpulet_status check_fc(int N, int In, int Out) {
    if (N < 1 || In < 1 || Out < 1) return GPULET_EINVAL;
    const long long lim = 1LL << 31;
    if (1LL * N * In >= lim || 1LL * Out * In >= lim || 1LL * N * Out >= lim) return GPULET_EINVAL;
    return GPULET_OK;
}

namespace {

// Long rows at serving batch sizes take fc_split_kernel: 64 outputs per workgroup and as many
// depth ranges (at most 8) as fill the gpu-let.
struct SplitPlan {
    bool wide;       // the layer takes fc_split_kernel
    int groups;      // output groups of 64 = one arrival counter each
    int ksplit;      // depth ranges wanted
    size_t need;     // bytes of partial tiles when ksplit > 1
};

SplitPlan plan_split(int N, int In, int Out, int n_cu) {
    SplitPlan s;
    s.wide = In >= 8192 && N <= 32;
    s.groups = (Out + 63) / 64;
    s.ksplit = s.wide ? std::max(1, std::min(8, (n_cu < 1 ? 1 : n_cu) / s.groups)) : 1;
    s.need = s.ksplit > 1 ? static_cast<size_t>(s.groups) * s.ksplit * (N <= 16 ? 1 : 2) * 4 * 64 * 16 : 0;
    return s;
}

// Scratch of the entry point that allocates nothing: partial tiles, then arrival counters.  One
// copy per GPU, held until the process ends; every call on a GPU shares it.
constexpr size_t kStaticTileBytes = 2u << 20;
constexpr int kStaticCounters = 1024;
static __device__ __align__(256) unsigned char scratch[kStaticTileBytes + kStaticCounters * sizeof(unsigned)];

constexpr int kMaxDevices = 64;
std::atomic<unsigned char *> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device, looked up once per device.
hipError_t static_scratch(unsigned char **out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    unsigned char *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(reinterpret_cast<void **>(&p), HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return hipSuccess;
}

__global__ void zero_counters_kernel(unsigned *cnt, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) cnt[i] = 0u;
}

}  // namespace

hipError_t launch_fc(const void *x, const void *w, const float *b, void *y, int N, int In, int Out,
                     int relu, int out_fp32, const LaunchCtx &ctx, hipStream_t stream) {
    FcParams p;
    p.x = static_cast<const __bf16 *>(x);
    p.w = static_cast<const __bf16 *>(w);
    p.b = b;
    p.y = y;
    p.N = N; p.In = In; p.Out = Out; p.relu = relu; p.out_fp32 = out_fp32;
    const bool vec = (In % 8 == 0) && (reinterpret_cast<uintptr_t>(x) % 16 == 0) &&
                     (reinterpret_cast<uintptr_t>(w) % 16 == 0);
    const bool wide = In >= 8192;  // long rows: 16 wavefronts per workgroup
    const SplitPlan plan = plan_split(N, In, Out, ctx.n_cu);
    if (plan.wide) {
        // The depth ranges need scratch for the partial tiles and one counter per output group,
        // otherwise there is one range.
        const int groups = plan.groups;
        const int steps = (In + 31) / 32;
        int ksplit = plan.ksplit;
        if (!ctx.scratch || !ctx.counters || groups > ctx.n_counters || plan.need > ctx.scratch_bytes) ksplit = 1;
        const int sps = (steps + ksplit - 1) / ksplit;
        const dim3 g(static_cast<unsigned>(groups), static_cast<unsigned>(ksplit));
#define GPULET_FC_SPLIT(NB, V) \
    hipLaunchKernelGGL((fc_split_kernel<NB, V>), g, dim3(1024), 0, stream, p, ctx.scratch, ctx.counters, ksplit, sps)
        if (N <= 16) { if (vec) GPULET_FC_SPLIT(1, true); else GPULET_FC_SPLIT(1, false); }
        else { if (vec) GPULET_FC_SPLIT(2, true); else GPULET_FC_SPLIT(2, false); }
#undef GPULET_FC_SPLIT
        return hipGetLastError();
    }
    const unsigned gx = static_cast<unsigned>((Out + 15) / 16);
    const dim3 grid(gx, N <= 16 ? 1u : static_cast<unsigned>((N + 31) / 32));
#define GPULET_FC_LAUNCH(NB, NW, V) \
    hipLaunchKernelGGL((fc_kernel<NB, NW, V>), grid, dim3(NW * 64), 0, stream, p)
    if (N <= 16) {
        if (wide) { if (vec) GPULET_FC_LAUNCH(1, 16, true); else GPULET_FC_LAUNCH(1, 16, false); }
        else { if (vec) GPULET_FC_LAUNCH(1, 4, true); else GPULET_FC_LAUNCH(1, 4, false); }
    } else {
        if (wide) { if (vec) GPULET_FC_LAUNCH(2, 16, true); else GPULET_FC_LAUNCH(2, 16, false); }
        else { if (vec) GPULET_FC_LAUNCH(2, 4, true); else GPULET_FC_LAUNCH(2, 4, false); }
    }
#undef GPULET_FC_LAUNCH
    return hipGetLastError();
}

// The same layer with the partial tiles and counters in the library's static device array
// instead of a gpu-let's allocation.  Nothing is allocated here or below: the array's address
// is looked up once per device, the counters are cleared by a small kernel on the caller's
// stream (a caller may be capturing the stream, and the array keeps what the last call left).
hipError_t launch_fc_static(const void *x, const void *w, const float *b, void *y, int N, int In, int Out,
                            int relu, int out_fp32, int n_cu, hipStream_t stream, bool *too_large) {
    *too_large = false;
    LaunchCtx ctx;
    ctx.n_cu = n_cu;
    const SplitPlan plan = plan_split(N, In, Out, n_cu);
    if (plan.wide && plan.ksplit > 1) {
        if (plan.need > kStaticTileBytes || plan.groups > kStaticCounters) {
            *too_large = true;
            return hipSuccess;
        }
        unsigned char *base = nullptr;
        const hipError_t e = static_scratch(&base);
        if (e != hipSuccess) return e;
        ctx.scratch = reinterpret_cast<float *>(base);
        ctx.scratch_bytes = kStaticTileBytes;
        ctx.counters = reinterpret_cast<unsigned *>(base + kStaticTileBytes);
        ctx.n_counters = kStaticCounters;
        hipLaunchKernelGGL(zero_counters_kernel, dim3((plan.groups + 255) / 256), dim3(256), 0, stream, ctx.counters,
                           plan.groups);
        const hipError_t le = hipGetLastError();
        if (le != hipSuccess) return le;
    }
    return launch_fc(x, w, b, y, N, In, Out, relu, out_fp32, ctx, stream);
}

}  // namespace gpulet
