// First layers of the image models (paper Sec. 5; Table 4): convolutions over at
// most four input channels.
#include "conv_common.h"

namespace gpulet {
namespace conv {

namespace {

// ---------------------------------------------------------------------------
// Image stems: C <= 4 (the RGB input of the ImageNet models, LeNet's single
// plane) with a filter of R x S, S <= 8.
//
// With so few channels a depth slice of the gathering kernels is mostly
// address arithmetic: every 2-byte element is located and fetched on its own.
// Here the depth is laid out as R filter rows of KROW = 16 or 32 elements, a
// filter row being S pixels of 4 channels (missing channels and pixels have
// zero weights).  In NHWC the S pixels a filter row touches are neighbours in
// memory, so once the input patch of a tile sits in LDS as 8-byte pixels
// (channels padded to 4), the fragment of output pixel q for filter row r and
// depth step j is 16 contiguous bytes at pixel q*stride + 4j + 2*(lane/32) of
// patch row r: no im2col copy is ever made.
//
// A workgroup is four wavefronts; each owns 32 consecutive output columns of
// one output row (tile = 4 rows x 32 columns of one image) and all BN = 32*NT
// filters, whose fragments it keeps in registers for its whole life while it
// walks over many tiles.  The layer is bound by instruction issue, not by the
// matrix cores (a tile is R*KROW/16*NT matrix instructions), so everything
// around them is kept short:
//  * loads are buffer loads whose offset is pushed out of range for padding,
//    missing channels and ragged tiles (they return zero): no branches;
//  * the patch is double buffered and requested two tiles ahead into
//    registers, so a tile has one workgroup barrier and never waits for memory;
//  * the product is taken as filters x pixels, which leaves every lane with
//    groups of 4 consecutive channels of one pixel; rounded to bf16 they cross
//    a piece of LDS private to the wavefront (no barrier) and return as 16
//    bytes per lane with eight consecutive lanes covering one pixel, so the
//    stores write whole 128-byte lines.  The accumulators start from the bias
//    (read from LDS) instead of zero.
// Needs a destination that allows aligned 16-byte stores, K % 8 == 0 and no
// residual operand; other layers stay with the gathering kernel.
// The depth is summed in ascending (r, s, c) order like every other kernel,
// but the sum starts from the bias and the zero padding changes how the terms
// group into matrix instructions, so results agree with the gathering kernel
// to rounding, not bit for bit; the choice of this kernel depends on the
// layer's shape and the destination's alignment only, never on the batch or
// the gpu-let.
// ---------------------------------------------------------------------------
constexpr int STEM_TP = 4, STEM_TQ = 32;   // output rows x columns per tile
constexpr int STEM_PX = 1024;              // input pixels a tile may touch (8 KB of LDS per buffer)
constexpr int STEM_PXT = STEM_PX / 256;    // ... per thread

template <int R, int KROW, int NT>
__global__ __launch_bounds__(256) void conv_stem_kernel(const ConvParams p, const int wgs_per_col, const int tiles_m,
                                                        const int tiles_q, const int tiles_pq) {
    fetch_params(p);
    constexpr int BN = NT * 32, KS = KROW / 16;
    constexpr int WELEMS = BN * R * KROW;  // padded weights, staged once on their way to registers
    constexpr int TROW = BN * 2 + 16;      // bytes per pixel row of the epilogue's transposition (padded)
    constexpr int STG_BYTES = WELEMS * 2 > 4 * 32 * TROW ? WELEMS * 2 : 4 * 32 * TROW;
    __shared__ __attribute__((aligned(16))) unsigned char stg_raw[STG_BYTES];
    __shared__ __attribute__((aligned(16))) uint2 patch[2][STEM_PX];
    __shared__ __attribute__((aligned(16))) float lbias[BN];

    const int col = blockIdx.x % p.tiles_n, j0 = blockIdx.x / p.tiles_n;
    const int n0 = col * BN;
    const int T = j0 < tiles_m ? (tiles_m - j0 + wgs_per_col - 1) / wgs_per_col : 0;  // uniform over the workgroup
    if (T == 0) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int frow = lane & 31, fhalf = lane >> 5;
    const int nrows = p.n_cb, ncols = p.tw;  // patch extent: 3*stride + R rows, 31*stride + KROW/4 pixels
    const int npx = nrows * ncols;

    const __amdgpu_buffer_rsrc_t rx =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<__bf16 *>(p.x), 0, p.x_bytes, RSRC_FLAGS);
    const __amdgpu_buffer_rsrc_t rw =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<__bf16 *>(p.w), 0, p.w_bytes, RSRC_FLAGS);

    // Weights -> LDS as [filter][r][s][4], zero where s >= S, c >= C or the filter does not exist.
    // Eight loads are issued before the first is used: one load-use chain per element would
    // cost a memory latency each, which is most of the life of a workgroup at small batches.
    {
        unsigned short *wl = reinterpret_cast<unsigned short *>(stg_raw);
        constexpr int WPT = (WELEMS + 255) / 256, WB = 8;
#pragma unroll
        for (int i0 = 0; i0 < WPT; i0 += WB) {
            unsigned short v[WB];
#pragma unroll
            for (int u = 0; u < WB; ++u) {
                const int i = tid + (i0 + u) * 256;
                const int f = i / (R * KROW), rem = i - f * (R * KROW);
                const int r = rem / KROW, kk = rem - r * KROW;
                const int sx = kk >> 2, c = kk & 3;
                const bool ok = i < WELEMS && n0 + f < p.K && sx < p.S && c < p.C;
                const unsigned off = ok ? static_cast<unsigned>(((((n0 + f) * R + r) * p.S + sx) * p.C + c) * 2) : OOB;
                v[u] = __builtin_amdgcn_raw_buffer_load_b16(rw, off, 0, 0);
            }
#pragma unroll
            for (int u = 0; u < WB; ++u) {
                const int i = tid + (i0 + u) * 256;
                if (i < WELEMS) wl[i] = v[u];
            }
        }
    }
    __syncthreads();
    bf16x8 wf[R][KS][NT];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int j = 0; j < KS; ++j)
#pragma unroll
            for (int t = 0; t < NT; ++t)
                wf[r][j][t] = *reinterpret_cast<const bf16x8 *>(stg_raw + 2 * ((t * 32 + frow) * (R * KROW) + r * KROW +
                                                                                 j * 16 + fhalf * 8));
    if (tid < BN) lbias[tid] = (p.b && n0 + tid < p.K) ? p.b[n0 + tid] : 0.f;

    // Tile t of this workgroup: image n, first output row p0 and column q0.
    struct Tile {
        int n, p0, q0;
    };
    auto tile_at = [&](int t) {
        const int tile = j0 + t * wgs_per_col;
        Tile r;
        r.n = fdiv(tile, p.d_pwt);
        const int rem = tile - r.n * tiles_pq;
        const int tp = fdiv(rem, p.d_ncb);
        r.p0 = tp * STEM_TP;
        r.q0 = (rem - tp * tiles_q) * STEM_TQ;
        return r;
    };
    // Patch pixels tid, tid + 256, ... of a tile, channels padded to four; zeros outside the
    // image.  Where a pixel sits inside the patch does not depend on the tile.
    const int iters = (npx + 255) >> 8;  // uniform
    int prow[STEM_PXT], pcol[STEM_PXT], poff[STEM_PXT];
#pragma unroll
    for (int i = 0; i < STEM_PXT; ++i) {
        const int px = tid + i * 256;
        prow[i] = fdiv(px, p.d_tw);
        pcol[i] = px - prow[i] * ncols;
        poff[i] = (prow[i] * p.W + pcol[i]) * p.C * 2;
        if (px >= npx) prow[i] = 1 << 28;  // never inside the image
    }
    auto fetch = [&](const Tile &tl, uint2 (&v)[STEM_PXT]) {
        const int h0 = tl.p0 * p.stride - p.pad, w0 = tl.q0 * p.stride - p.pad;
        const int base = ((tl.n * p.H + h0) * p.W + w0) * p.C * 2;  // may be negative; only used where in range
#pragma unroll
        for (int i = 0; i < STEM_PXT; ++i) {
            if (i >= iters) break;
            const bool ok = static_cast<unsigned>(h0 + prow[i]) < static_cast<unsigned>(p.H) &&
                            static_cast<unsigned>(w0 + pcol[i]) < static_cast<unsigned>(p.W);
            const unsigned off = ok ? static_cast<unsigned>(base + poff[i]) : OOB;
            if (p.C == 4) {  // pixels are 8 bytes already (an 8-byte aligned tensor is checked on the host)
                const auto two = __builtin_amdgcn_raw_buffer_load_b64(rx, off, 0, 0);
                v[i] = make_uint2(two[0], two[1]);
                continue;
            }
            unsigned e[4];
#pragma unroll
            for (int c = 0; c < 4; ++c)
                e[c] = c < p.C ? static_cast<unsigned>(__builtin_amdgcn_raw_buffer_load_b16(rx, off + 2 * c, 0, 0)) : 0u;
            v[i] = make_uint2(e[0] | (e[1] << 16), e[2] | (e[3] << 16));
        }
    };
    auto stash = [&](int buf, const uint2 (&v)[STEM_PXT]) {
#pragma unroll
        for (int i = 0; i < STEM_PXT; ++i) {
            if (i >= iters) break;
            if (tid + i * 256 < npx) patch[buf][tid + i * 256] = v[i];
        }
    };

    // Registers -> memory for one wavefront's 32 pixels x BN filters.  Accumulator register v of
    // a lane belongs to filter 8*(v/4) + 4*(lane/32) + v%4 of its 32 and to pixel lane%32, so a
    // lane holds 8-byte pieces of one pixel.  They pass through a region of LDS private to the
    // wavefront (rows of TROW bytes per pixel; no workgroup barrier) and come back with eight
    // consecutive lanes holding the eight 16-byte groups of one pixel: every store instruction
    // then writes whole 128-byte lines.
    auto store_rows = [&](const Tile &tl, const f32x16 (&acc)[NT]) {
        unsigned char *tr = stg_raw + wave * (32 * TROW);
        const unsigned limit = relu_limit(p.relu);
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                *reinterpret_cast<uint2 *>(tr + frow * TROW + t * 64 + g * 16 + fhalf * 8) =
                    make_uint2(relu_or_pass(pack_bf16(acc[t][4 * g], acc[t][4 * g + 1]), limit),
                               relu_or_pass(pack_bf16(acc[t][4 * g + 2], acc[t][4 * g + 3]), limit));
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        constexpr int GPP = BN / 8;        // 16-byte groups per pixel
        constexpr int PPI = 64 / GPP;      // pixels per store instruction
        const int grp = lane % GPP, px0 = lane / GPP;
        const int pp = tl.p0 + wave;
        const int k = n0 + grp * 8;
        const int mrow = (tl.n * p.P + pp) * p.Q;
        uint4 out[32 / PPI];
#pragma unroll
        for (int i = 0; i < 32 / PPI; ++i)
            out[i] = *reinterpret_cast<const uint4 *>(tr + (px0 + i * PPI) * TROW + grp * 16);
#pragma unroll
        for (int i = 0; i < 32 / PPI; ++i) {
            const int qq = tl.q0 + px0 + i * PPI;
            if (pp < p.P && qq < p.Q && k < p.K)
                *reinterpret_cast<uint4 *>(p.y + ((mrow + qq) * p.ldy + p.y_off + k)) = out[i];
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };

    // The patch of tile t+1 is written to LDS during tile t and was requested during tile t-1:
    // a tile is too short to hide a memory latency itself.
    uint2 nxt[STEM_PXT], nxt2[STEM_PXT];
    Tile cur = tile_at(0), nx = cur;
    fetch(cur, nxt);
    stash(0, nxt);  // (the first barrier of the tile loop also frees the weights' staging area)
    if (T > 1) {
        nx = tile_at(1);
        fetch(nx, nxt);
    }
    // One tile: `have` holds the patch of tile t+1, `want` receives that of tile t+2 (the two
    // register sets swap roles every tile, so no copy has to wait for a load).
    auto one_tile = [&](int t, const uint2 (&have)[STEM_PXT], uint2 (&want)[STEM_PXT]) {
        // Patch buffer t&1 is complete, and nobody reads buffer (t+1)&1 any more.
        __syncthreads();
        Tile nx2 = nx;
        if (t + 2 < T) {
            nx2 = tile_at(t + 2);
            fetch(nx2, want);
        }
        f32x16 acc[NT];
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 b4 = *reinterpret_cast<const float4 *>(&lbias[j * 32 + 8 * g + 4 * fhalf]);
                acc[j][4 * g] = b4.x;
                acc[j][4 * g + 1] = b4.y;
                acc[j][4 * g + 2] = b4.z;
                acc[j][4 * g + 3] = b4.w;
            }
        const uint2 *pbuf = patch[t & 1] + (wave * p.stride) * ncols + frow * p.stride + fhalf * 2;
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int j = 0; j < KS; ++j) {
                const int sx = j * 4 + fhalf * 2;  // filter column of this lane's first pixel
                const uint2 *pa = pbuf + r * ncols + j * 4;
                uint2 lo = pa[0], hi = pa[1];
                // Pixels past the filter's width meet zero weights; clear them so that a
                // non-finite neighbour cannot turn 0 * x into NaN.
                if (sx >= p.S) lo = make_uint2(0u, 0u);
                if (sx + 1 >= p.S) hi = make_uint2(0u, 0u);
                union {
                    uint4 u;
                    bf16x8 h;
                } a;
                a.u = make_uint4(lo.x, lo.y, hi.x, hi.y);
#pragma unroll
                for (int n = 0; n < NT; ++n)
                    acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[r][j][n], a.h, acc[n], 0, 0, 0);
            }
        if (t + 1 < T) stash((t + 1) & 1, have);
        store_rows(cur, acc);
        cur = nx;
        nx = nx2;
    };
    for (int t = 0; t < T; t += 2) {
        one_tile(t, nxt, nxt2);
        if (t + 1 < T) one_tile(t + 1, nxt2, nxt);
    }
}

// One instance of the stem kernel: workgroups per CU the hardware can hold (asked once per
// instance; registers bound it, the weights of a 7 x 7 x 64 filter bank alone take 112) and the
// launch.  Every workgroup of the grid is resident at once and walks its share of the tiles.
template <int R, int KROW, int NT>
hipError_t launch_stem_rkn(ConvParams p, int n_cu, int tiles_m, int tiles_q, int tiles_pq, hipStream_t stream) {
    static const int per_cu = [] {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, conv_stem_kernel<R, KROW, NT>, 256, 0) != hipSuccess || n < 1)
            n = 1;
        return n;
    }();
    const int wgs_per_col = std::max(1, std::min(tiles_m, per_cu * n_cu / p.tiles_n));
    hipLaunchKernelGGL((conv_stem_kernel<R, KROW, NT>), dim3(static_cast<unsigned>(wgs_per_col * p.tiles_n)), dim3(256),
                       0, stream, p, wgs_per_col, tiles_m, tiles_q, tiles_pq);
    return hipGetLastError();
}

template <int R, int KROW>
hipError_t launch_stem_r(const ConvParams &p, int n_cu, int tiles_m, int tiles_q, int tiles_pq, hipStream_t stream) {
    if (p.K <= 32) return launch_stem_rkn<R, KROW, 1>(p, n_cu, tiles_m, tiles_q, tiles_pq, stream);
    return launch_stem_rkn<R, KROW, 2>(p, n_cu, tiles_m, tiles_q, tiles_pq, stream);
}

}  // namespace

// The stem kernel: at most four channels, a filter row of at most eight pixels, 3, 5 or 7
// filter rows, a tile's input patch within the staged limit, 16-byte stores possible, no residual.
bool stem_applicable(const ConvParams &p) {
    if (p.C > 4 || p.ldx != p.C || p.S > 8 || !(p.R == 3 || p.R == 5 || p.R == 7)) return false;
    if (!p.vec_store || p.K % 8 != 0 || p.res) return false;
    if (p.C == 4 && reinterpret_cast<uintptr_t>(p.x) % 8 != 0) return false;  // 8-byte pixel loads
    const int krow = p.S <= 4 ? 16 : 32;
    const int nrows = (STEM_TP - 1) * p.stride + p.R, ncols = (STEM_TQ - 1) * p.stride + krow / 4;
    return nrows * ncols <= STEM_PX;
}

hipError_t launch_stem(ConvParams p, int n_cu, hipStream_t stream) {
    const int krow = p.S <= 4 ? 16 : 32;
    const int bn = p.K <= 32 ? 32 : 64;
    const int tiles_p = (p.P + STEM_TP - 1) / STEM_TP, tiles_q = (p.Q + STEM_TQ - 1) / STEM_TQ;
    const int tiles_pq = tiles_p * tiles_q;
    const int tiles_m = p.N * tiles_pq;
    p.tiles_n = (p.K + bn - 1) / bn;
    p.n_tiles = tiles_m * p.tiles_n;
    p.split_k = 1;
    p.n_cb = (STEM_TP - 1) * p.stride + p.R;         // patch rows
    p.tw = (STEM_TQ - 1) * p.stride + krow / 4;      // patch pixels per row
    p.d_tw = make_fastdiv(p.tw);
    p.d_pwt = make_fastdiv(tiles_pq);
    p.d_ncb = make_fastdiv(tiles_q);
    if (p.R == 3 && krow == 16) return launch_stem_r<3, 16>(p, n_cu, tiles_m, tiles_q, tiles_pq, stream);
    if (p.R == 3) return launch_stem_r<3, 32>(p, n_cu, tiles_m, tiles_q, tiles_pq, stream);
    if (p.R == 5 && krow == 16) return launch_stem_r<5, 16>(p, n_cu, tiles_m, tiles_q, tiles_pq, stream);
    if (p.R == 5) return launch_stem_r<5, 32>(p, n_cu, tiles_m, tiles_q, tiles_pq, stream);
    if (krow == 16) return launch_stem_r<7, 16>(p, n_cu, tiles_m, tiles_q, tiles_pq, stream);
    return launch_stem_r<7, 32>(p, n_cu, tiles_m, tiles_q, tiles_pq, stream);
}

}  // namespace conv
}  // namespace gpulet
