// What the max-pool kernel and kernels that carry a max pool as a side job share
// (paper Sec. 5: pooling layers of the served models): the parameters and the
// work of one thread.
#pragma once

#include <hip/hip_runtime.h>

#include "device_util.h"

namespace gpulet {

struct PoolParams {
    const __bf16 *x;
    __bf16 *y;
    int N, C, H, W, P, Q, k, stride, pad;
    int total;  // work items
    FastDiv d_cv, d_q, d_p;  // pool_max_item: divisions by C/8, Q and P
};

// Work item idx (< p.total) of a K x K max pool: 8 consecutive channels of one output pixel.
template <int K>
__device__ __forceinline__ void pool_max_item(const PoolParams &p, int idx) {
    const int cv = p.C >> 3;
    int t = fdiv(idx, p.d_cv);
    const int c8 = idx - t * cv;
    const int t1 = fdiv(t, p.d_q);
    const int q = t - t1 * p.Q;
    const int n = fdiv(t1, p.d_p);
    const int pp = t1 - n * p.P;
    const int h0 = pp * p.stride - p.pad, w0 = q * p.stride - p.pad;
    int rowo[K], colo[K];
#pragma unroll
    for (int d = 0; d < K; ++d) {
        rowo[d] = (n * p.H + min(max(h0 + d, 0), p.H - 1)) * p.W * p.C + c8 * 8;
        colo[d] = min(max(w0 + d, 0), p.W - 1) * p.C;
    }
    uint4 v[K * K];
#pragma unroll
    for (int r = 0; r < K; ++r)
#pragma unroll
        for (int sx = 0; sx < K; ++sx) v[r * K + sx] = *reinterpret_cast<const uint4 *>(p.x + rowo[r] + colo[sx]);
    unsigned k[4] = {bf16_pair_order_key(v[0].x), bf16_pair_order_key(v[0].y), bf16_pair_order_key(v[0].z), bf16_pair_order_key(v[0].w)};
#pragma unroll
    for (int j = 1; j < K * K; ++j) {
        k[0] = max_keys(k[0], bf16_pair_order_key(v[j].x));
        k[1] = max_keys(k[1], bf16_pair_order_key(v[j].y));
        k[2] = max_keys(k[2], bf16_pair_order_key(v[j].z));
        k[3] = max_keys(k[3], bf16_pair_order_key(v[j].w));
    }
    *reinterpret_cast<uint4 *>(p.y + (((n * p.P + pp) * p.Q + q) * p.C + c8 * 8)) =
        make_uint4(bf16_pair_order_key(k[0]), bf16_pair_order_key(k[1]), bf16_pair_order_key(k[2]), bf16_pair_order_key(k[3]));
}

}  // namespace gpulet
