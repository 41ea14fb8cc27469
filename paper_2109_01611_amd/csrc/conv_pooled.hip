// Pooling branch of an inception block in one kernel (paper Sec. 5; GoogLeNet of
// Table 4).
#include "conv_common.h"

namespace gpulet {
namespace conv {

namespace {

// ---------------------------------------------------------------------------
// Max pool 3x3 / stride 1 / pad 1 followed by a 1x1 convolution (the pooling
// branch of an inception block), in one kernel: the pooled tensor is never
// written.  The pool kernel alone took about as long as the small projection
// that follows it (9-12 us against 6-8 us at batch 32), most of it fixed cost.
//
// Same 64 x 64 tile, depth order and epilogue as the gathering kernel, so the
// result is bit-identical to pooling and convolving separately.  What differs
// is the loader of the pixel operand: for each 16-byte chunk (8 channels of one
// pixel) a thread loads the nine window pixels - coordinates clamped to the
// image, which repeats taps that are in the window anyway, so padding never
// wins - and keeps their maximum.  bf16 are sign-magnitude; x ^ ((x >> 15) &
// 0x7fff) per 16-bit half maps them to integers in the same order (and back),
// so the maximum is four packed 16-bit integer instructions per tap.  The raw
// loads of depth slice j+1 are issued before the matrix instructions of slice j
// and reduced after them.
// ---------------------------------------------------------------------------
constexpr int PC_BM = 32, PC_BN = 64;

// These layers are small (a few hundred pixel tiles at most) and all latency: a tile is 32
// pixels x 64 filters so that there are enough workgroups, every thread pools one chunk per
// slice, and the raw loads of slices j+1 and j+2 are in flight while slice j is multiplied.
// Only two of the four wavefronts issue matrix instructions (32 x 32 each); all four load.
__global__ __launch_bounds__(256) void pooled_conv1x1_kernel(const ConvParams p) {
    fetch_params(p);
    constexpr int BM = PC_BM, BN = PC_BN, LDT = BN + 8;
    constexpr int STAGE = (BM + BN) * BK;  // elements per LDS stage: pixel rows, then filter rows
    constexpr int LDS_ELEMS = 2 * STAGE > BM * LDT * 2 ? 2 * STAGE : BM * LDT * 2;
    __shared__ __attribute__((aligned(16))) __bf16 lds[LDS_ELEMS];

    const int tile = tile_of_block(p);
    if (tile >= p.n_tiles) return;
    const int tm = fdiv(tile, p.d_tiles_n), tn = tile - tm * p.tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;
    const BiasRegs bias_regs = load_bias<BN, 256>(p, n0);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int frow = lane & 31, fhalf = lane >> 5;
    const int cc = tid & 7, lrow = tid >> 3;  // this thread fills chunk cc of pixel row lrow and filter rows lrow, lrow + 32

    // Element offsets of the three window rows and columns of this thread's pixel (clamped).
    int rowo[3], colo[3];
    const bool m_ok = m0 + lrow < p.M;
    {
        const int mm = m_ok ? m0 + lrow : 0;
        const int n = fdiv(mm, p.d_pq);
        const int pq = mm - n * (p.H * p.W);
        const int h = fdiv(pq, p.d_q), w = pq - h * p.W;
#pragma unroll
        for (int d = 0; d < 3; ++d) {
            rowo[d] = (n * p.H + min(max(h + d - 1, 0), p.H - 1)) * p.W * p.C;
            colo[d] = min(max(w + d - 1, 0), p.W - 1) * p.C;
        }
    }
    int b_base[2];
    bool b_ok[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int k = n0 + lrow + 32 * i;
        b_ok[i] = k < p.K;
        b_base[i] = (b_ok[i] ? k : 0) * p.C;
    }
    struct Raw {
        uint4 a[9], b[2];
    };
    const int nk = (p.C + BK - 1) / BK;
    auto load_slice = [&](int kt, Raw &r) {
        const int c0 = kt * BK + cc * CHUNK;
        const bool c_ok = kt < nk && c0 < p.C;  // C % 8 == 0: a chunk is inside the depth or past it as a whole
#pragma unroll
        for (int t = 0; t < 9; ++t)
            r.a[t] = (c_ok && m_ok) ? *reinterpret_cast<const uint4 *>(p.x + rowo[t / 3] + colo[t % 3] + c0)
                                    : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int i = 0; i < 2; ++i)
            r.b[i] = (c_ok && b_ok[i]) ? *reinterpret_cast<const uint4 *>(p.w + b_base[i] + c0) : make_uint4(0u, 0u, 0u, 0u);
    };
    auto store_slice = [&](int buf, const Raw &r) {
        __bf16 *sA = lds + buf * STAGE, *sB = sA + BM * BK;
        unsigned k[4] = {bf16_pair_order_key(r.a[0].x), bf16_pair_order_key(r.a[0].y), bf16_pair_order_key(r.a[0].z),
                         bf16_pair_order_key(r.a[0].w)};
#pragma unroll
        for (int t = 1; t < 9; ++t) {
            k[0] = max_keys(k[0], bf16_pair_order_key(r.a[t].x));
            k[1] = max_keys(k[1], bf16_pair_order_key(r.a[t].y));
            k[2] = max_keys(k[2], bf16_pair_order_key(r.a[t].z));
            k[3] = max_keys(k[3], bf16_pair_order_key(r.a[t].w));
        }
        *reinterpret_cast<uint4 *>(&sA[lds_pos(lrow, cc)]) = make_uint4(
            bf16_pair_order_key(k[0]), bf16_pair_order_key(k[1]), bf16_pair_order_key(k[2]), bf16_pair_order_key(k[3]));
#pragma unroll
        for (int i = 0; i < 2; ++i) *reinterpret_cast<uint4 *>(&sB[lds_pos(lrow + 32 * i, cc)]) = r.b[i];
    };

    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    // Slice kt: reduce and store its raw loads, barrier, request slice kt+2 into the registers
    // just freed, multiply.  The two register sets swap roles every slice.
    auto one_slice = [&](int kt, Raw &mine) {
        store_slice(kt & 1, mine);
        __syncthreads();  // stage kt&1 is complete; nobody reads it for slice kt-2 any more
        load_slice(kt + 2, mine);
        if (wave < 2) {
            const __bf16 *sA = lds + (kt & 1) * STAGE, *sB = sA + BM * BK;
#pragma unroll
            for (int ks = 0; ks < BK / 16; ++ks) {
                const bf16x8 fa = *reinterpret_cast<const bf16x8 *>(&sA[lds_pos(frow, ks * 2 + fhalf)]);
                const bf16x8 fb = *reinterpret_cast<const bf16x8 *>(&sB[lds_pos(wave * 32 + frow, ks * 2 + fhalf)]);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc, 0, 0, 0);
            }
        }
    };
    Raw r0, r1;
    load_slice(0, r0);
    load_slice(1, r1);
    for (int kt = 0; kt < nk; kt += 2) {
        one_slice(kt, r0);
        if (kt + 1 < nk) one_slice(kt + 1, r1);
    }
    __syncthreads();  // the last stage has been read: the fp32 tile may overwrite the stages
    float *stg = reinterpret_cast<float *>(lds);
    if (wave < 2) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = 8 * (v >> 2) + 4 * fhalf + (v & 3);
            stg[row * LDT + wave * 32 + frow] = acc[v];
        }
    }
    __syncthreads();
    finish_tile<BM, BN, 256>(p, stg, n0, bias_regs, [&](int row) { return m0 + row < p.M ? m0 + row : -1; });
}

}  // namespace

hipError_t launch_pooled_conv(ConvParams p, hipStream_t stream) {
    const int tiles_m = (p.M + PC_BM - 1) / PC_BM;
    p.tiles_n = (p.K + PC_BN - 1) / PC_BN;
    p.n_tiles = tiles_m * p.tiles_n;
    p.split_k = 1;
    p.d_tiles_n = make_fastdiv(p.tiles_n);
    p.tiles_per_xcd = (p.n_tiles + 7) / 8;
    hipLaunchKernelGGL(pooled_conv1x1_kernel, dim3(static_cast<unsigned>(p.tiles_per_xcd * 8)), dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace conv
}  // namespace gpulet
