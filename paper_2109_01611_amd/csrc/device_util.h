// Small device-side helpers shared by the layer kernels of this library: the
// multiply-shift division, packed bf16 rounding and ReLU, and the integer keys
// that order bf16 values.  Device code; include from .hip files only.
#ifndef GPULET_DEVICE_UTIL_H
#define GPULET_DEVICE_UTIL_H

#include <hip/hip_runtime.h>

namespace gpulet {

typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) short s16x2;

// Division of a non-negative int below 2^30 by a fixed positive divisor through one 64-bit
// multiply: q = (n * mul) >> shift with shift = 30 + ceil(log2 d), mul = floor(2^shift / d) + 1.
// Exact because n * (mul * d - 2^shift) <= n * d < 2^shift.  Index arithmetic in these kernels is
// full of divisions by layer constants; the compiler's general sequence costs about 25
// instructions each, on the critical path before the first load can be issued.
struct FastDiv {
    unsigned mul;
    int shift;
};

inline FastDiv make_fastdiv(int d) {
    int lg = 0;
    while ((1LL << lg) < d) ++lg;
    FastDiv f;
    f.shift = 30 + lg;
    f.mul = static_cast<unsigned>((1ULL << f.shift) / static_cast<unsigned long long>(d) + 1ULL);
    return f;
}

__device__ __forceinline__ int fdiv(int n, const FastDiv f) {
    return static_cast<int>((static_cast<unsigned long long>(static_cast<unsigned>(n)) * f.mul) >> f.shift);
}

// Two floats -> two bf16 (round to nearest even) in one dword, the first in the low half.
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
    const f32x2 v = {lo, hi};
    const bf16x2 h = __builtin_convertvector(v, bf16x2);
    return *reinterpret_cast<const unsigned *>(&h);
}

// ReLU on a pair of bf16 in one dword, switched without a branch: as signed 16-bit integers
// every negative bf16 (and -0) is below zero, so max(bits, 0) is max(x, +0); with the limit at
// 0x8000 the operation is the identity.  Rounding to bf16 keeps the sign, so clamping after the
// rounding gives the same bits as clamping the fp32 value before it.
__device__ __forceinline__ unsigned relu_limit(int relu) { return relu ? 0u : 0x80008000u; }
__device__ __forceinline__ unsigned relu_or_pass(unsigned pair, unsigned limit) {
    const s16x2 r = __builtin_elementwise_max(*reinterpret_cast<const s16x2 *>(&pair),
                                              *reinterpret_cast<const s16x2 *>(&limit));
    return *reinterpret_cast<const unsigned *>(&r);
}

// bf16 are sign-magnitude: x ^ ((x >> 15) & 0x7fff) per 16-bit half maps a pair of them to two
// signed integers in the same order, and back (the map is its own inverse).  The maximum of
// bf16 values is then a packed 16-bit integer maximum: exact, without unpacking to fp32.
__device__ __forceinline__ unsigned bf16_pair_order_key(unsigned v) {
    const s16x2 x = *reinterpret_cast<const s16x2 *>(&v);
    const s16x2 k = x ^ ((x >> 15) & static_cast<short>(0x7fff));
    return *reinterpret_cast<const unsigned *>(&k);
}
__device__ __forceinline__ unsigned max_keys(unsigned a, unsigned b) {
    const s16x2 r = __builtin_elementwise_max(*reinterpret_cast<const s16x2 *>(&a), *reinterpret_cast<const s16x2 *>(&b));
    return *reinterpret_cast<const unsigned *>(&r);
}

}  // namespace gpulet
#endif  // GPULET_DEVICE_UTIL_H
