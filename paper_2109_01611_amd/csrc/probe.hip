// Placement probe: records on which die and compute unit the hardware ran
// each workgroup of a launch, to check that a gpu-let's CU mask (paper
// Sec. 2.3: a gpu-let owns a fraction of the GPU's compute) is honoured.
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

}  // namespace

hipError_t launch_probe(uint32_t *out, int n_blocks, hipStream_t stream) {
    hipLaunchKernelGGL(probe_kernel, dim3(static_cast<unsigned>(n_blocks)), dim3(64), 0, stream, out,
                       n_blocks);
    return hipGetLastError();
}

}  // namespace gpulet
