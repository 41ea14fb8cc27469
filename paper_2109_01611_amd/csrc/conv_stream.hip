// Streaming kernel for 1x1 convolutions with a short depth (paper Sec. 5; the
// first stage of ResNet-50, MobileNet's pointwise layers).
#include "conv_common.h"

namespace gpulet {
namespace conv {

namespace {

// ---------------------------------------------------------------------------
// 1x1 filters over 64 or 128 input channels with many output tiles: a streaming
// kernel.
//
// Such a layer moves far more bytes than it multiplies (one or two depth slices
// per tile), and with one tile per workgroup its three phases - waiting for the
// loads, multiplying, and the epilogue's LDS round trip and stores - run one
// after the other on every CU, roughly in lockstep across the chip.  Here a
// workgroup keeps its BN x C slab of the weights in LDS and walks over many
// pixel tiles of BM = 64 rows; its producer wavefronts run two tiles ahead, so
// the input of tiles t+1 and t+2 is in flight while the consumers multiply and
// store tile t.  The fp32 staging tile of the epilogue has LDS of its own (the
// ring is busy), and only the consumers take part in the epilogue: a producer's
// explicit transfer counting must not be mixed with stores.
//
// Every wavefront executes the same two barriers per tile:
//   B1(t): the input of tile t has landed (each producer waited for its own
//          transfers; only those of tile t+1 may still be in flight), and every
//          consumer has finished the epilogue of tile t-1, so the staging tile
//          and the ring stage of tile t-1 are free.  Producers then refill that
//          stage with tile t+2; consumers multiply tile t and park the result.
//   B2(t): the staging tile is complete; consumers run the epilogue.
// The number of tiles of a workgroup is computed before the roles split, so both
// roles always execute the same number of barriers.
// The depth order is that of the kernels above, so results are bit-identical.
// ---------------------------------------------------------------------------
constexpr int STREAM_BM = 64, STREAM_BN = 128;

template <int NK>
__global__ __launch_bounds__(12 * 64) void conv1x1_stream_kernel(const ConvParams p, const int wgs_per_col,
                                                                 const int tiles_m) {
    fetch_params(p);
    constexpr int BM = STREAM_BM, BN = STREAM_BN, NCONS = 8, NPROD = 4, NA = 3;
    constexpr int CWN = 4, WM = 32, WN = 32;                 // consumers: 2 x 4 wavefronts of 32 x 32
    constexpr int PROWS = NPROD * 8;                          // 32 tile rows per round of producer instructions
    constexpr int AINS = BM / PROWS, WINS = BN / PROWS;       // transfers per lane: per slice of a tile / of the slab
    constexpr int AOPS = NK * AINS;                           // transfers per lane and tile
    constexpr int ASTAGE = NK * BM * BK, WSLAB = NK * BN * BK;
    constexpr int LDT = BN + 8;
    static_assert(NK * WINS + 2 * AOPS <= 63, "6-bit transfer counter");
    __shared__ __attribute__((aligned(1024))) __bf16 wlds[WSLAB];
    __shared__ __attribute__((aligned(1024))) __bf16 alds[NA * ASTAGE];
    __shared__ __attribute__((aligned(16))) float stg[BM * LDT];

    // Workgroup (col, j) owns channel tile `col` and pixel tiles j, j + wgs_per_col, ...
    const int col = blockIdx.x % p.tiles_n, j0 = blockIdx.x / p.tiles_n;
    const int n0 = col * BN;
    const int T = j0 < tiles_m ? (tiles_m - j0 + wgs_per_col - 1) / wgs_per_col : 0;  // uniform over the workgroup
    if (T == 0) return;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    if (wave >= NCONS) {
        // ------------------------------------------------------------ producer
        const int pw = wave - NCONS;
        const i32x4 rx = make_rsrc(p.x, p.x_bytes);
        const i32x4 rw = make_rsrc(p.w, p.w_bytes);
        const int lrow = pw * 8 + (lane >> 3);
        const int cc = (lane & 7) ^ ((lrow >> 1) & 7);  // logical chunk this lane fetches (same for rows 32 apart)

        // weights: slice q, rows i*PROWS + lrow
#pragma unroll
        for (int q = 0; q < NK; ++q)
#pragma unroll
            for (int i = 0; i < WINS; ++i) {
                const int k = n0 + i * PROWS + lrow;
                // chunks past the last channel (C below a whole number of slices) read as zeros
                const bool in = k < p.K && q * BK + cc * CHUNK < p.C;
                const unsigned off = in ? static_cast<unsigned>((k * p.C + q * BK + cc * CHUNK) * 2) : OOB;
                dma16(rw, lds_addr(wlds + q * BN * BK) + (i * PROWS + pw * 8) * (BK * 2), off);
            }
        auto issue_tile = [&](int t) {
            const int m0 = (j0 + t * wgs_per_col) * BM;
            const unsigned base = lds_addr(alds + (t % NA) * ASTAGE) + pw * 8 * (BK * 2);
#pragma unroll
            for (int i = 0; i < AINS; ++i) {
                const int m = m0 + i * PROWS + lrow;
                unsigned pix = OOB;
                if (t < T && m < p.M) {
                    const int n = fdiv(m, p.d_pq);
                    const int pq = m - n * (p.P * p.Q);
                    const int pp = fdiv(pq, p.d_q), qq = pq - pp * p.Q;
                    pix = static_cast<unsigned>((((n * p.H + pp * p.stride) * p.W + qq * p.stride) * p.C + cc * CHUNK) * 2);
                }
#pragma unroll
                for (int q = 0; q < NK; ++q)
                    dma16(rx, base + (q * BM + i * PROWS) * (BK * 2),
                          (pix == OOB || q * BK + cc * CHUNK >= p.C) ? OOB : pix + q * (BK * 2));
            }
        };
        issue_tile(0);
        issue_tile(1);
        for (int t = 0; t < T; ++t) {
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(AOPS));  // all but the transfers of tile t+1 have landed
            __syncthreads();                              // B1
            issue_tile(t + 2);
            __syncthreads();                              // B2
        }
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    } else {
        // ------------------------------------------------------------ consumer
        const BiasRegs bias_regs = load_bias<BN, NCONS * 64>(p, n0);
        const int wy = wave / CWN, wx = wave - wy * CWN;
        const int frow = lane & 31, fhalf = lane >> 5;
        for (int t = 0; t < T; ++t) {
            const int m0 = (j0 + t * wgs_per_col) * BM;
            __syncthreads();                              // B1
            const __bf16 *sA = alds + (t % NA) * ASTAGE;
            f32x16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
            for (int q = 0; q < NK; ++q)
#pragma unroll
                for (int ks = 0; ks < BK / 16; ++ks) {
                    const bf16x8 fa = *reinterpret_cast<const bf16x8 *>(
                        &sA[q * BM * BK + lds_pos(wy * WM + frow, ks * 2 + fhalf)]);
                    const bf16x8 fb = *reinterpret_cast<const bf16x8 *>(
                        &wlds[q * BN * BK + lds_pos(wx * WN + frow, ks * 2 + fhalf)]);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc, 0, 0, 0);
                }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = wy * WM + 8 * (v >> 2) + 4 * fhalf + (v & 3);
                stg[row * LDT + wx * WN + frow] = acc[v];
            }
            __syncthreads();                              // B2
            finish_tile<BM, BN, NCONS * 64>(p, stg, n0, bias_regs,
                                            [&](int row) { return m0 + row < p.M ? m0 + row : -1; });
        }
    }
}

}  // namespace

// The streaming 1x1 kernel: at most 128 input channels (one or two depth slices, the last one
// possibly partial), unit filter.
bool stream_applicable(const ConvParams &p, bool vec) {
    return vec && p.ldx == p.C && p.k2 == p.K && !p.side_pool.y && p.R == 1 && p.S == 1 && p.pad == 0 && p.C <= 2 * BK;
}

// Chosen automatically for one depth slice (C <= 64: two workgroups per CU) and at least four tiles
// per CU, where it measured 11 % faster than the best one-tile-per-workgroup tile (1x1 64->256 on
// 56x56 at batch 32: 20.3 -> 18.0 us).  With two slices (C up to 128) it only pays when a single
// filter tile is walked over very many pixel tiles (128->128 on 75x75 at batch 32: 21.0 -> 17.7 us,
// on 56x56 13.6 -> 12.9 us); with more filter tiles it measured 8-15 % slower.
bool stream_eligible(const ConvParams &p, bool vec, int n_cu) {
    const long long tiles_n = (p.K + STREAM_BN - 1) / STREAM_BN;
    const long long tiles = 1LL * ((p.M + STREAM_BM - 1) / STREAM_BM) * tiles_n;
    if (!stream_applicable(p, vec)) return false;
    return p.C <= BK ? tiles >= 4LL * n_cu : (tiles_n == 1 && tiles >= 6LL * n_cu);
}

hipError_t launch_stream(ConvParams p, int n_cu, hipStream_t stream) {
    const int tiles_m = (p.M + STREAM_BM - 1) / STREAM_BM;
    p.tiles_n = (p.K + STREAM_BN - 1) / STREAM_BN;
    p.n_tiles = tiles_m * p.tiles_n;
    p.split_k = 1;
    // two workgroups per CU with one depth slice (75 KB of LDS each), one with two (115 KB)
    const int slots = n_cu * (p.C <= BK ? 2 : 1);
    const int wgs_per_col = std::max(1, std::min(tiles_m, slots / p.tiles_n));
    const dim3 grid(static_cast<unsigned>(wgs_per_col * p.tiles_n));
    if (p.C <= BK)
        hipLaunchKernelGGL(conv1x1_stream_kernel<1>, grid, dim3(12 * 64), 0, stream, p, wgs_per_col, tiles_m);
    else
        hipLaunchKernelGGL(conv1x1_stream_kernel<2>, grid, dim3(12 * 64), 0, stream, p, wgs_per_col, tiles_m);
    return hipGetLastError();
}

}  // namespace conv
}  // namespace gpulet
