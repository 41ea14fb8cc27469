// Placement probe: records on which die and compute unit the hardware ran
// each workgroup of a launch, to check that a gpu-let's CU mask (paper
// Sec. 2.3: a gpu-let owns a fraction of the GPU's compute) is honoured.
// Rate probe: what the matrix pipelines sustain on a gpu-let, by operand pattern
// (the ceiling against which the convolution kernels' utilisation is read).
#include <hip/hip_runtime.h>

#include "gpulet_internal.h"

namespace gpulet {
namespace {

__global__ __launch_bounds__(64) void probe_kernel(uint32_t *out, int n_blocks) {
    unsigned xcc, hw;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
    // Spin a little so workgroups spread over every CU the mask allows instead
    // of all retiring on the first few.
    const long long t0 = wall_clock64();
    while (wall_clock64() - t0 < 2000) {
    }
    if (threadIdx.x == 0 && static_cast<int>(blockIdx.x) < n_blocks) {
        out[2 * blockIdx.x] = xcc;
        out[2 * blockIdx.x + 1] = hw;
    }
}

// Rate probe: nothing but matrix instructions on register operands, to measure what the matrix
// pipelines sustain at the clock the power limit allows for a given operand pattern.  Every
// wavefront holds eight A and eight B fragments and runs all 64 pairs per loop iteration into
// four accumulators in rotation (an accumulator is reused every fourth instruction, past the
// instruction's latency).  dense != 0: fragments are pseudo-random bf16 in (-1, 1), different in
// every lane and register; dense == 0: all zero.
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 probe_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float probe_f32x16;

__device__ __forceinline__ unsigned probe_hash(unsigned v) {
    v ^= v >> 16;
    v *= 0x7feb352dU;
    v ^= v >> 15;
    v *= 0x846ca68bU;
    v ^= v >> 16;
    return v;
}

__global__ __launch_bounds__(512) void mfma_rate_kernel(float *out, int iters, int dense) {
    probe_bf16x8 a[8], b[8];
    const unsigned tid = blockIdx.x * blockDim.x + threadIdx.x;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const unsigned ha = probe_hash(tid * 131u + i * 8u + e), hb = probe_hash(~tid * 137u + i * 8u + e);
            const float fa = dense ? static_cast<float>(ha & 0xffff) * (1.0f / 32768.0f) - 1.0f : 0.0f;
            const float fb = dense ? static_cast<float>(hb & 0xffff) * (1.0f / 32768.0f) - 1.0f : 0.0f;
            a[i][e] = static_cast<__bf16>(fa);
            b[i][e] = static_cast<__bf16>(fb);
        }
    probe_f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j)
                acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[j & 3], 0, 0, 0);
    }
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) sum += acc[j][v];
    out[tid] = sum;
}

}  // namespace

hipError_t launch_mfma_rate(float *out, int blocks, int waves, int iters, int dense, hipStream_t stream) {
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(static_cast<unsigned>(blocks)), dim3(static_cast<unsigned>(waves * 64)), 0,
                       stream, out, iters, dense);
    return hipGetLastError();
}

hipError_t launch_probe(uint32_t *out, int n_blocks, hipStream_t stream) {
    hipLaunchKernelGGL(probe_kernel, dim3(static_cast<unsigned>(n_blocks)), dim3(64), 0, stream, out,
                       n_blocks);
    return hipGetLastError();
}

}  // namespace gpulet
