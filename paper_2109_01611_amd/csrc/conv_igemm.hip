// Convolution layer of the forward pass served on a gpu-let (paper Sec. 5; the
// models of Table 4), as an implicit GEMM on gfx950 matrix cores:
//
//   rows    m = (n, p, q)   output pixels          M  = N*P*Q
//   columns k               output channels        Ng = K
//   depth   g = (r, s, c)   filter taps x channels Kg = R*S*C
//
// x is NHWC and w is KRSC, so both operands are contiguous along the depth
// and neither the im2col matrix nor a transposed weight is ever built.
//
// One workgroup owns a BM x BN output tile and walks the depth in slices of 64.
// Its wavefronts are specialised.  Producer wavefronts only compute addresses
// and issue 16-byte buffer loads (8 channels of one tap) that land directly in
// LDS without passing through registers; the hardware range check of the
// buffer descriptor returns zeros for padding taps and ragged edges, so the
// gather has no branches.  Consumer wavefronts only read 8-element fragments
// back from the XOR-swizzled LDS tile with ds_read_b128 and feed
// v_mfma_f32_32x32x16_bf16; accumulators stay in registers for the whole
// depth.  Slices travel through a ring of three LDS stages, two loads ahead of
// the one being multiplied, with one workgroup barrier per slice.  When the
// channel count is a multiple of 64 the depth is walked with the filter taps
// innermost, so a producer's lane keeps its channel offset and only steps the
// tap.  The epilogue parks the fp32 tile in the idle ring, adds bias and the
// optional residual, applies ReLU, rounds once to bf16 and writes 16-byte
// rows, optionally at a channel offset inside a wider (concatenated) tensor.
// Optionally several workgroups share a tile by splitting the depth; partial
// tiles meet in device scratch and the last one to arrive reduces them in a
// fixed order.
//
// Channel counts that are not multiples of 8 (image stems, LeNet) take a
// scalar-gather variant of the same tiling with four wavefronts.
#include <climits>

#include "conv_common.h"

namespace gpulet {
namespace conv {

namespace {

// Epilogue shared by both kernels.  Accumulator register v of a lane holds row
// 8*(v/4) + 4*(lane/32) + v%4 and column lane%32 of its 32x32 tile.
template <int MT, int NT>
__device__ __forceinline__ void store_tile(const ConvParams &p, const f32x16 (&acc)[MT][NT], int m_base,
                                           int n_base, int lane) {
    const int frow = lane & 31, fhalf = lane >> 5;
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int k = n_base + j * 32 + frow;
        if (k >= p.K) continue;
        const float bias = p.b ? p.b[k] : 0.f;
#pragma unroll
        for (int i = 0; i < MT; ++i) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m_base + i * 32 + 8 * (v >> 2) + 4 * fhalf + (v & 3);
                if (m >= p.M) continue;
                float val = acc[i][j][v] + bias;
                if (p.res) val += static_cast<float>(p.res[m * p.K + k]);
                if (p.relu) val = val > 0.f ? val : 0.f;
                p.y[m * p.ldy + p.y_off + k] = static_cast<__bf16>(val);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Main kernel: C % 8 == 0.  POINTWISE = 1x1 filter without padding (no bounds
// tests at all; a strided 1x1 is pointwise too).
//
// Staging uses buffer loads that write straight into LDS (no registers, no
// ds_write): one wavefront instruction moves 64 x 16 bytes into a contiguous
// 1 KB span = 8 tile rows of 128 bytes, lane i landing at byte 16*i.  The XOR
// swizzle is therefore applied on the global side: the lane that fills
// physical chunk q of row t fetches logical chunk q ^ swizzle(t).  Offsets
// past the buffer make the hardware write zeros (padding, ragged edges).
// NS LDS stages form a ring: while slice j is multiplied, slices j+1 .. j+NS-1
// are in flight.
// ---------------------------------------------------------------------------

// Wavefronts are specialised.  The first CWM x CWN wavefronts ("consumers")
// only read LDS and issue MFMAs; the last NPROD wavefronts ("producers") only
// compute addresses and issue transfers.  A wavefront blocked on a saturated
// memory pipeline therefore never holds back matrix instructions.  Every ring
// step has one workgroup barrier: before it a producer waits for its own
// transfers of slice j, after it the stage slice j-1 occupied is free again.
// EXTRA: the layer has a second destination or a pooling side job (1x1 layers only); layers
// without either run the instance that knows of neither.
template <int BM, int BN, int CWM, int CWN, int NPROD, int NS, bool POINTWISE, bool EXTRA>
__device__ __forceinline__ void conv_igemm_body(const ConvParams &p, const int bid) {
    constexpr int NCONS = CWM * CWN;
    constexpr int WM = BM / CWM, WN = BN / CWN;  // consumer wavefront tile
    constexpr int MT = WM / 32, NT = WN / 32;    // MFMA tiles per consumer
    static_assert(MT >= 1 && NT >= 1 && WM % 32 == 0 && WN % 32 == 0, "tile shape");
    static_assert(NPROD == 2 || NPROD == 4, "swizzle key must not depend on the instruction index");
    constexpr int PROWS = NPROD * 8;                       // tile rows one round of producer instructions fills
    constexpr int AINS = BM / PROWS, BINS = BN / PROWS;    // transfers per producer lane and slice
    static_assert(BM % PROWS == 0 && BN % PROWS == 0, "tile rows per producer round");
    constexpr int STAGE = (BM + BN) * BK;                  // elements per LDS stage: A rows, then B rows
    static_assert(NS >= 2 && (AINS + BINS) * (NS - 2) <= 63, "ring depth vs the 6-bit transfer counter");

    constexpr int LDT = BN + 8;  // padded row of the fp32 epilogue tile that reuses the ring
    constexpr int RING = NS * STAGE > BM * LDT * 2 ? NS * STAGE : BM * LDT * 2;
    __shared__ __attribute__((aligned(1024))) __bf16 ring[RING];

    // Split-K: consecutive work items share an output tile and each takes a
    // contiguous range of depth slices.
    // Workgroups past the tiles carry the layer's side job, if it has one: a max pool of the same
    // input, which would otherwise be a launch of its own with nothing but fixed cost to it.
    // They are told apart inside the early exit that idle workgroups take anyway, so that a
    // workgroup with a tile does not wait for one more field of the argument block first.
    fetch_params(p);
    const int item = tile_of_block(p, bid);
    if (item >= p.n_tiles * p.split_k || bid >= p.tiles_per_xcd * 8) {
        if (EXTRA && bid >= p.tiles_per_xcd * 8 && p.side_blocks > 0) {
            const int idx = (bid - p.tiles_per_xcd * 8) * ((CWM * CWN + NPROD) * 64) + static_cast<int>(threadIdx.x);
            if (idx < p.side_pool.total) pool_max_item<3>(p.side_pool, idx);
        }
        return;
    }
    const int tile = fdiv(item, p.d_split_k), ks = item - tile * p.split_k;
    const int tm = fdiv(tile, p.d_tiles_n), tn = tile - tm * p.tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;
    const BiasRegs bias_regs = load_bias<BN, (CWM * CWN + NPROD) * 64>(p, n0);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nk_all = (p.Kg + BK - 1) / BK;
    const int k_first = ks * p.sps;                                  // first slice of this workgroup
    const int nk = max(0, min(nk_all, k_first + p.sps) - k_first);  // slices of this workgroup

    f32x16 acc[MT][NT];  // consumers only

    if (wave >= NCONS) {
        // ------------------------------------------------------------ producer
        const int pw = wave - NCONS;
        const i32x4 rx = make_rsrc(p.x, p.x_bytes);
        const i32x4 rw = make_rsrc(p.w, p.w_bytes);

        // Instruction u of this wavefront fills tile rows u*PROWS + pw*8 .. +8;
        // this lane fills physical chunk lane&7 of row u*PROWS + lrow, i.e.
        // fetches logical chunk cc (the same for every u).
        const int lrow = pw * 8 + (lane >> 3);
        const int cc = (lane & 7) ^ ((lrow >> 1) & 7);

        // Byte offset of tap (0, 0), channel 0 of each pixel row (may be negative
        // before the tap offset is added), and the pixel's top-left corner.
        int a_off[AINS], a_h0[AINS], a_w0[AINS];
#pragma unroll
        for (int i = 0; i < AINS; ++i) {
            const int m = m0 + lrow + PROWS * i;
            if (m < p.M) {
                const int n = fdiv(m, p.d_pq);
                const int pq = m - n * (p.P * p.Q);
                const int pp = fdiv(pq, p.d_q), qq = pq - pp * p.Q;
                a_h0[i] = pp * p.stride - p.pad;
                a_w0[i] = qq * p.stride - p.pad;
                a_off[i] = (((n * p.H + a_h0[i]) * p.W + a_w0[i]) * p.ldx) * 2;
            } else {
                a_h0[i] = -(1 << 28);  // fails every bounds test
                a_w0[i] = -(1 << 28);
                a_off[i] = static_cast<int>(OOB);
            }
        }
        unsigned b_off[BINS];
#pragma unroll
        for (int i = 0; i < BINS; ++i) {
            const int k = n0 + lrow + PROWS * i;
            b_off[i] = k < p.K ? static_cast<unsigned>((k * p.Kg + cc * CHUNK) * 2) : OOB;
        }

        // Depth position of the chunk this lane fetches next: element index g, its
        // filter tap (r, s), channel c, and the tap's byte offset inside the image.
        // With dense pixels (ldx == C) advancing s by one and c by -C leaves the
        // address unchanged (a filter row covers a contiguous span of the image row),
        // so the offset only jumps when the filter moves to its next row; when the
        // layer reads a channel slice of wider pixels it also skips ldx - C elements
        // from one pixel to the next.
        //
        // Two depth orders.  Linear: g runs through (r, s, c) as the weights are
        // stored.  Tap-inner (C a multiple of 64, filter larger than 1x1): for each
        // block of 64 channels all taps follow one another, so the image rows a
        // workgroup just fetched for one tap are fetched again for the next while
        // they are still in the nearest cache.  Both operands use the same order,
        // so only the summation order of the result changes.
        int g, r, s, c, tap, cblk = 0, issued = 0;
        if (!POINTWISE && p.tap_inner) {
            const int rs = p.R * p.S;
            const int cb = k_first / rs, t = k_first - cb * rs;
            r = fdiv(t, p.d_s);
            s = t - r * p.S;
            cblk = cb * BK;
            c = cblk + cc * CHUNK;
            g = t * p.C + c;
            tap = ((r * p.W + s) * p.ldx + c) * 2;
        } else {
            g = k_first * BK + cc * CHUNK;
            const int t = fdiv(g, p.d_c);
            c = g - t * p.C;
            r = fdiv(t, p.d_s);
            s = t - r * p.S;
            tap = ((r * p.W + s) * p.ldx + c) * 2;
        }
        auto normalise = [&]() {
            while (c >= p.C) {
                c -= p.C;
                tap += (p.ldx - p.C) * 2;  // nothing when the pixels are dense
                if (++s == p.S) {
                    s = 0;
                    ++r;
                    tap += (p.W - p.S) * p.ldx * 2;
                }
            }
        };

        // Starts the transfer of the next depth slice into `stage` and advances the
        // position.  Slices past the end of the depth transfer zeros nobody reads.
        auto issue_next = [&](const __bf16 *stage) {
            const bool g_ok = issued < nk && g < p.Kg;
            unsigned base = lds_addr(stage) + pw * 8 * (BK * 2);
#pragma unroll
            for (int i = 0; i < AINS; ++i) {
                bool ok = g_ok;
                if (!POINTWISE)
                    ok = ok & ((unsigned)(a_h0[i] + r) < (unsigned)p.H) & ((unsigned)(a_w0[i] + s) < (unsigned)p.W);
                const unsigned off = ok ? static_cast<unsigned>(a_off[i] + tap) : OOB;
                dma16(rx, base + i * PROWS * (BK * 2), off);
            }
            base += BM * (BK * 2);
#pragma unroll
            for (int i = 0; i < BINS; ++i) {
                const unsigned off = g_ok ? b_off[i] + static_cast<unsigned>(g - cc * CHUNK) * 2u : OOB;
                dma16(rw, base + i * PROWS * (BK * 2), off);
            }
            ++issued;
            if (!POINTWISE && p.tap_inner) {
                g += p.C;
                tap += p.ldx * 2;
                if (++s == p.S) {
                    s = 0;
                    tap += (p.W - p.S) * p.ldx * 2;
                    if (++r == p.R) {
                        r = 0;
                        cblk += BK;
                        g = cblk + cc * CHUNK;
                        tap = g * 2;
                    }
                }
            } else {
                g += BK;
                c += BK;
                tap += BK * 2;
                if (!POINTWISE) normalise();
            }
        };

        // Step j: wait for this lane's transfers of slice j (those of the NS-2 later
        // slices may stay in flight), meet everybody, refill the stage slice j-1 was
        // read from with slice j+NS-1.
#pragma unroll
        for (int i = 0; i < NS - 1; ++i) issue_next(ring + i * STAGE);
        auto step = [&](int refill) {
            __builtin_amdgcn_s_waitcnt(vmcnt_imm((AINS + BINS) * (NS - 2)));
            __syncthreads();
            issue_next(ring + refill * STAGE);
        };
        // The ring position is a compile-time constant inside the unrolled body.
        int kt = 0;
        for (; kt + NS <= nk; kt += NS) {
#pragma unroll
            for (int u = 0; u < NS; ++u) step((u + NS - 1) % NS);
        }
#pragma unroll
        for (int u = 0; u < NS - 1; ++u)
            if (kt + u < nk) step((u + NS - 1) % NS);
        // Every transfer has landed before the ring is reused by the epilogue.
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    } else {
    // ---------------------------------------------------------------- consumer
    const int wy = wave / CWN, wx = wave - wy * CWN;
    const int frow = lane & 31;   // row of an MFMA operand this lane supplies
    const int fhalf = lane >> 5;  // which 8 of the 16 depth elements of a step

#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    auto step = [&](int cur) {
        __syncthreads();
        const __bf16 *sA = ring + cur * STAGE, *sB = sA + BM * BK;
        constexpr int KS = BK / 16;
        if constexpr (MT * NT == 1) {
            // One matrix instruction per pair of fragment reads: the wavefront would wait out the
            // LDS latency before each of them.  All reads of the slice are issued first, and the
            // scheduling barrier keeps them there; each matrix instruction then waits only for its
            // own operands, and the compiler moves the next slice's barrier and reads up between
            // this slice's last matrix instructions.  (With more accumulators per wavefront the
            // extra fragment registers cost more than the latency: measured slower.)
            bf16x8 fa[KS], fb[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                fa[ks] = *reinterpret_cast<const bf16x8 *>(&sA[lds_pos(wy * WM + frow, ks * 2 + fhalf)]);
                fb[ks] = *reinterpret_cast<const bf16x8 *>(&sB[lds_pos(wx * WN + frow, ks * 2 + fhalf)]);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks], fb[ks], acc[0][0], 0, 0, 0);
        } else {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                bf16x8 fa[MT], fb[NT];
#pragma unroll
                for (int i = 0; i < MT; ++i)
                    fa[i] = *reinterpret_cast<const bf16x8 *>(&sA[lds_pos(wy * WM + i * 32 + frow, ks * 2 + fhalf)]);
#pragma unroll
                for (int j = 0; j < NT; ++j)
                    fb[j] = *reinterpret_cast<const bf16x8 *>(&sB[lds_pos(wx * WN + j * 32 + frow, ks * 2 + fhalf)]);
#pragma unroll
                for (int i = 0; i < MT; ++i)
#pragma unroll
                    for (int j = 0; j < NT; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
            }
        }
    };
    int kt = 0;
    for (; kt + NS <= nk; kt += NS) {
#pragma unroll
        for (int u = 0; u < NS; ++u) step(u);
    }
#pragma unroll
    for (int u = 0; u < NS - 1; ++u)
        if (kt + u < nk) step(u);

    }

    // ------------------------------------------------------------------ epilogue
    // The accumulators hold one column (channel) and 16 scattered rows per lane,
    // which would mean 2-byte stores.  They go through LDS instead: consumers
    // drop acc + bias as fp32 into the (now idle) ring, then every wavefront of
    // the workgroup picks up 8 consecutive channels of a pixel, adds the
    // residual, applies ReLU, rounds once to bf16 and stores 16 bytes.
    // Rows are padded by 8 floats so that lanes 32..63 (4 rows further down) use
    // the other half of the banks.
    float *stg = reinterpret_cast<float *>(ring);
    __syncthreads();  // all LDS reads of the main loop are done, all transfers have landed
    if (wave < NCONS) {
        const int wy = wave / CWN, wx = wave - wy * CWN;
        const int frow = lane & 31, fhalf = lane >> 5;
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const int col = wx * WN + j * 32 + frow;
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = wy * WM + i * 32 + 8 * (v >> 2) + 4 * fhalf + (v & 3);
                    stg[row * LDT + col] = acc[i][j][v];
                }
        }
    }
    __syncthreads();
    constexpr int NTHR = (NCONS + NPROD) * 64;
    constexpr int VPR = BN / 8;  // 8-channel groups per tile row

    // Split-K: every workgroup but the last to arrive parks its partial tile in
    // scratch and leaves; the last one adds the others' tiles to its own, always
    // in split order so the sum does not depend on who came last.  Arrival is
    // counted with one atomic per workgroup; nobody ever waits.
    //
    // The dies' L2 caches are not coherent with one another, and a device-wide
    // fence would write back and invalidate a whole L2.  So the partial tiles and
    // the counter are accessed with device-scope (cache-bypassing) loads and
    // stores only, and a workgroup waits for its own stores to be acknowledged
    // before it counts itself in.
    if (p.split_k > 1) {
        constexpr int DEVICE_SCOPE = 16;  // cache policy sc1: device scope, bypasses the die-local caches
        const __amdgpu_buffer_rsrc_t rp = __builtin_amdgcn_make_buffer_rsrc(
            p.part, 0, p.n_tiles * p.split_k * (BM * BN * 4), RSRC_FLAGS);
        const int mine = (tile * p.split_k + ks) * (BM * BN * 4);  // byte offset of this workgroup's tile
        for (int it = threadIdx.x; it < BM * VPR; it += NTHR) {
            const int row = it / VPR, cv = it - row * VPR;
            const u32x4 lo = *reinterpret_cast<const u32x4 *>(&stg[row * LDT + cv * 8]);
            const u32x4 hi = *reinterpret_cast<const u32x4 *>(&stg[row * LDT + cv * 8 + 4]);
            __builtin_amdgcn_raw_buffer_store_b128(lo, rp, mine + (row * BN + cv * 8) * 4, 0, DEVICE_SCOPE);
            __builtin_amdgcn_raw_buffer_store_b128(hi, rp, mine + (row * BN + cv * 8 + 4) * 4, 0, DEVICE_SCOPE);
        }
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // this lane's partial-tile stores have reached memory
        __syncthreads();
        __shared__ unsigned arrived;
        if (threadIdx.x == 0) {
            arrived = __hip_atomic_fetch_add(&p.cnt[tile], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (arrived == static_cast<unsigned>(p.split_k - 1))  // ready for the next launch
                __hip_atomic_store(&p.cnt[tile], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        if (arrived != static_cast<unsigned>(p.split_k - 1)) return;
        const int base = tile * p.split_k * (BM * BN * 4);
        constexpr int ITEMS = (BM * VPR + NTHR - 1) / NTHR;  // 8-channel groups per thread
        float sum[ITEMS][8];
#pragma unroll
        for (int i = 0; i < ITEMS; ++i)
#pragma unroll
            for (int e = 0; e < 8; ++e) sum[i][e] = 0.f;
        for (int q = 0; q < p.split_k; ++q) {
            u32x4 a[ITEMS], b[ITEMS];
#pragma unroll
            for (int i = 0; i < ITEMS; ++i) {  // all loads of one partial tile in flight together
                const int it = threadIdx.x + i * NTHR;
                const int row = it / VPR, cv = it - row * VPR;
                const int off = it < BM * VPR ? base + q * (BM * BN * 4) + (row * BN + cv * 8) * 4 : static_cast<int>(OOB);
                a[i] = __builtin_amdgcn_raw_buffer_load_b128(rp, off, 0, DEVICE_SCOPE);
                b[i] = __builtin_amdgcn_raw_buffer_load_b128(rp, off + 16, 0, DEVICE_SCOPE);
            }
#pragma unroll
            for (int i = 0; i < ITEMS; ++i)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    sum[i][e] += __uint_as_float(a[i][e]);
                    sum[i][4 + e] += __uint_as_float(b[i][e]);
                }
        }
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const int it = threadIdx.x + i * NTHR;
            if (it < BM * VPR) {
                const int row = it / VPR, cv = it - row * VPR;
#pragma unroll
                for (int e = 0; e < 8; ++e) stg[row * LDT + cv * 8 + e] = sum[i][e];
            }
        }
        // each thread re-reads only what it wrote itself, in the same iteration order
    }
    finish_tile<BM, BN, NTHR, EXTRA>(p, stg, n0, bias_regs, [&](int row) { return m0 + row < p.M ? m0 + row : -1; });
}

template <int BM, int BN, int CWM, int CWN, int NPROD, int NS, bool POINTWISE, bool EXTRA = false>
__global__ __launch_bounds__((CWM * CWN + NPROD) * 64) void conv_igemm_kernel(const ConvParams p) {
    conv_igemm_body<BM, BN, CWM, CWN, NPROD, NS, POINTWISE, EXTRA>(p, blockIdx.x);
}

// Several independent layers in one launch (branches of an inception block, a projection
// shortcut next to the first layer of its block): each workgroup finds the layer its block
// index falls into and runs that layer's tile as above.  The general instance serves 1x1
// members too (its bounds tests always pass for them); when every member is 1x1 the instance
// without bounds tests is used.  Either way a member's results are the bits of its own launch.
template <int BM, int BN, int CWM, int CWN, int NPROD, int NS, bool POINTWISE>
__global__ __launch_bounds__((CWM * CWN + NPROD) * 64) void conv_igemm_group_kernel(const ConvGroup g) {
    const int b = blockIdx.x;
    int j = 0;
#pragma unroll
    for (int i = 1; i < MAX_GROUP; ++i)
        if (b >= g.first[i]) j = i;
    conv_igemm_body<BM, BN, CWM, CWN, NPROD, NS, POINTWISE, false>(g.p[j], b - g.first[j]);
}

// ---------------------------------------------------------------------------
// Any channel count: every element of a chunk is decoded and loaded on its own.
// Used by the image stems (C = 3) and LeNet (C = 1, 6); one slice of prefetch.
// ---------------------------------------------------------------------------
template <int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(NTHREADS) void conv_igemm_any_kernel(const ConvParams p) {
    static_assert(WGM * WGN == 4, "four wavefronts per workgroup");
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int MT = WM / 32, NT = WN / 32;
    constexpr int AROWS = BM / 32, BROWS = BN / 32;

    __shared__ __attribute__((aligned(16))) __bf16 sA[2][BM * BK];
    __shared__ __attribute__((aligned(16))) __bf16 sB[2][BN * BK];

    const int tile = tile_of_block(p);
    if (tile >= p.n_tiles) return;
    const int tm = tile / p.tiles_n, tn = tile - tm * p.tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wy = wave / WGN, wx = wave - wy * WGN;
    const int cc = tid & 7;
    const int lrow = tid >> 3;

    int a_base[AROWS], a_h0[AROWS], a_w0[AROWS];
#pragma unroll
    for (int i = 0; i < AROWS; ++i) {
        const int m = m0 + lrow + 32 * i;
        if (m < p.M) {
            const int n = m / (p.P * p.Q);
            const int pq = m - n * (p.P * p.Q);
            const int pp = pq / p.Q, qq = pq - pp * p.Q;
            a_h0[i] = pp * p.stride - p.pad;
            a_w0[i] = qq * p.stride - p.pad;
            a_base[i] = ((n * p.H + a_h0[i]) * p.W + a_w0[i]) * p.ldx;
        } else {
            a_h0[i] = -(1 << 28);
            a_w0[i] = -(1 << 28);
            a_base[i] = 0;
        }
    }
    int b_base[BROWS];
    bool b_ok[BROWS];
#pragma unroll
    for (int i = 0; i < BROWS; ++i) {
        const int k = n0 + lrow + 32 * i;
        b_ok[i] = k < p.K;
        b_base[i] = (b_ok[i] ? k : 0) * p.Kg;
    }

    uint4 ra[AROWS], rb[BROWS];
    const unsigned short *xs = reinterpret_cast<const unsigned short *>(p.x);
    const unsigned short *ws = reinterpret_cast<const unsigned short *>(p.w);

    auto load_slice = [&](int kt) {
        const int g0 = kt * BK + cc * CHUNK;
        int rs = g0 / p.C;
        int c = g0 - rs * p.C;
        int r = rs / p.S, s = rs - r * p.S;
        unsigned short ea[AROWS][CHUNK], eb[BROWS][CHUNK];
#pragma unroll
        for (int e = 0; e < CHUNK; ++e) {
            const bool g_ok = g0 + e < p.Kg;
            const int tap = (r * p.W + s) * p.ldx + c;
#pragma unroll
            for (int i = 0; i < AROWS; ++i) {
                const bool ok = g_ok && (unsigned)(a_h0[i] + r) < (unsigned)p.H &&
                                (unsigned)(a_w0[i] + s) < (unsigned)p.W;
                ea[i][e] = ok ? xs[a_base[i] + tap] : (unsigned short)0;
            }
#pragma unroll
            for (int i = 0; i < BROWS; ++i)
                eb[i][e] = (g_ok && b_ok[i]) ? ws[b_base[i] + g0 + e] : (unsigned short)0;
            if (++c == p.C) {
                c = 0;
                if (++s == p.S) {
                    s = 0;
                    ++r;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < AROWS; ++i)
            ra[i] = make_uint4(ea[i][0] | ((unsigned)ea[i][1] << 16), ea[i][2] | ((unsigned)ea[i][3] << 16),
                               ea[i][4] | ((unsigned)ea[i][5] << 16), ea[i][6] | ((unsigned)ea[i][7] << 16));
#pragma unroll
        for (int i = 0; i < BROWS; ++i)
            rb[i] = make_uint4(eb[i][0] | ((unsigned)eb[i][1] << 16), eb[i][2] | ((unsigned)eb[i][3] << 16),
                               eb[i][4] | ((unsigned)eb[i][5] << 16), eb[i][6] | ((unsigned)eb[i][7] << 16));
    };

    auto store_slice = [&](int buf) {
#pragma unroll
        for (int i = 0; i < AROWS; ++i) *reinterpret_cast<uint4 *>(&sA[buf][lds_pos(lrow + 32 * i, cc)]) = ra[i];
#pragma unroll
        for (int i = 0; i < BROWS; ++i) *reinterpret_cast<uint4 *>(&sB[buf][lds_pos(lrow + 32 * i, cc)]) = rb[i];
    };

    f32x16 acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nk = (p.Kg + BK - 1) / BK;
    const int frow = lane & 31, fhalf = lane >> 5;

    load_slice(0);
    store_slice(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_slice(kt + 1);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fa[MT], fb[NT];
#pragma unroll
            for (int i = 0; i < MT; ++i)
                fa[i] = *reinterpret_cast<const bf16x8 *>(&sA[buf][lds_pos(wy * WM + i * 32 + frow, ks * 2 + fhalf)]);
#pragma unroll
            for (int j = 0; j < NT; ++j)
                fb[j] = *reinterpret_cast<const bf16x8 *>(&sB[buf][lds_pos(wx * WN + j * 32 + frow, ks * 2 + fhalf)]);
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) store_slice(buf ^ 1);
        __syncthreads();
    }

    store_tile<MT, NT>(p, acc, m0 + wy * WM, n0 + wx * WN, lane);
}

// CWM x CWN consumers and NPROD producers for the main kernel; the scalar-gather
// kernel always runs four wavefronts as WGM x WGN.
template <int BM, int BN, int CWM, int CWN, int NPROD, int NS, int WGM, int WGN>
hipError_t launch_tile(ConvParams p, bool vec, int split_k, hipStream_t stream) {
    const int tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.K + BN - 1) / BN;
    p.n_tiles = tiles_m * p.tiles_n;
    const int nk = (p.Kg + BK - 1) / BK;
    p.split_k = vec ? split_k : 1;
    p.d_tiles_n = make_fastdiv(p.tiles_n);
    p.d_split_k = make_fastdiv(p.split_k);
    p.sps = (nk + p.split_k - 1) / p.split_k;
    p.tiles_per_xcd = (p.n_tiles * p.split_k + 7) / 8;  // work items per die
    const bool pointwise = p.R == 1 && p.S == 1 && p.pad == 0;
    constexpr int THREADS = (CWM * CWN + NPROD) * 64;
    p.side_blocks = (vec && pointwise && p.side_pool.y) ? (p.side_pool.total + THREADS - 1) / THREADS : 0;
    if (p.side_pool.y && !p.side_blocks) return hipErrorInvalidValue;  // nobody would compute the pool
    const dim3 grid(static_cast<unsigned>(p.tiles_per_xcd * 8 + p.side_blocks));
    const dim3 block(THREADS);
    if (vec && pointwise && (p.side_blocks > 0 || p.k2 < p.K))
        hipLaunchKernelGGL((conv_igemm_kernel<BM, BN, CWM, CWN, NPROD, NS, true, true>), grid, block, 0, stream, p);
    else if (vec && pointwise)
        hipLaunchKernelGGL((conv_igemm_kernel<BM, BN, CWM, CWN, NPROD, NS, true>), grid, block, 0, stream, p);
    else if (vec)
        hipLaunchKernelGGL((conv_igemm_kernel<BM, BN, CWM, CWN, NPROD, NS, false>), grid, block, 0, stream, p);
    else
        hipLaunchKernelGGL((conv_igemm_any_kernel<BM, BN, WGM, WGN>), grid, dim3(NTHREADS), 0, stream, p);
    return hipGetLastError();
}

template <int BM, int BN, int CWM, int CWN, int NPROD, int NS>
hipError_t launch_group_tile(const ConvParams *ps, int n, hipStream_t stream) {
    ConvGroup g;
    int blocks = 0;
    bool pointwise = true;
    for (int j = 0; j < n; ++j) pointwise = pointwise && ps[j].R == 1 && ps[j].S == 1 && ps[j].pad == 0;
    for (int j = 0; j < MAX_GROUP; ++j) {
        g.first[j] = j < n ? blocks : INT_MAX;
        g.p[j] = ps[j < n ? j : 0];
        if (j >= n) continue;
        ConvParams &p = g.p[j];
        const int tiles_m = (p.M + BM - 1) / BM;
        p.tiles_n = (p.K + BN - 1) / BN;
        p.n_tiles = tiles_m * p.tiles_n;
        p.split_k = 1;
        p.d_tiles_n = make_fastdiv(p.tiles_n);
        p.d_split_k = make_fastdiv(1);
        p.sps = (p.Kg + BK - 1) / BK;
        p.tiles_per_xcd = (p.n_tiles + 7) / 8;
        p.side_blocks = 0;
        blocks += p.tiles_per_xcd * 8;
    }
    g.first[MAX_GROUP] = INT_MAX;
    const dim3 grid(static_cast<unsigned>(blocks)), block((CWM * CWN + NPROD) * 64);
    if (pointwise)
        hipLaunchKernelGGL((conv_igemm_group_kernel<BM, BN, CWM, CWN, NPROD, NS, true>), grid, block, 0, stream, g);
    else
        hipLaunchKernelGGL((conv_igemm_group_kernel<BM, BN, CWM, CWN, NPROD, NS, false>), grid, block, 0, stream, g);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_igemm_group(const ConvParams *p, int n, int tile, bool two_stage, hipStream_t stream) {
    if (n < 2 || n > MAX_GROUP) return hipErrorInvalidValue;
    switch (tile) {
        case 0:
            if (two_stage) return launch_group_tile<128, 128, 4, 2, 4, 2>(p, n, stream);
            return launch_group_tile<128, 128, 4, 2, 4, 3>(p, n, stream);
        case 1: return launch_group_tile<128, 64, 4, 2, 4, 3>(p, n, stream);
        case 2: return launch_group_tile<64, 128, 2, 4, 4, 3>(p, n, stream);
        case 3: return launch_group_tile<64, 64, 2, 2, 2, 3>(p, n, stream);
        case 4: return launch_group_tile<128, 32, 4, 1, 2, 3>(p, n, stream);
        case 5: return launch_group_tile<32, 128, 1, 4, 2, 3>(p, n, stream);
        case 12: return launch_group_tile<192, 128, 2, 4, 4, 3>(p, n, stream);
        case 13: return launch_group_tile<96, 128, 1, 4, 4, 3>(p, n, stream);
        default: return launch_group_tile<256, 128, 4, 2, 4, 3>(p, n, stream);
    }
}

hipError_t launch_igemm(const ConvParams &p, bool vec, int tile, int split_k, bool two_stage, hipStream_t stream) {
    switch (tile) {
        case 0:
            // With more tiles than CUs, a two-stage ring (64 KB, two workgroups per CU, one's loads
            // overlapping the other's epilogue) beats the deeper prefetch of three stages.
            if (two_stage && split_k == 1) return launch_tile<128, 128, 4, 2, 4, 2, 2, 2>(p, vec, 1, stream);
            return launch_tile<128, 128, 4, 2, 4, 3, 2, 2>(p, vec, split_k, stream);
        case 1: return launch_tile<128, 64, 4, 2, 4, 3, 2, 2>(p, vec, split_k, stream);
        case 2: return launch_tile<64, 128, 2, 4, 4, 3, 2, 2>(p, vec, split_k, stream);
        case 3: return launch_tile<64, 64, 2, 2, 2, 3, 2, 2>(p, vec, split_k, stream);
        case 4: return launch_tile<128, 32, 4, 1, 2, 3, 4, 1>(p, vec, split_k, stream);
        case 5: return launch_tile<32, 128, 1, 4, 2, 3, 1, 4>(p, vec, split_k, stream);
        // three row tiles per consumer (96 pixels x 32 filters); the scalar-gather variant has no such
        // instance and takes the nearest shape
        case 12:
            if (!vec) return launch_tile<256, 128, 4, 2, 4, 3, 2, 2>(p, vec, split_k, stream);
            return launch_tile<192, 128, 2, 4, 4, 3, 2, 2>(p, vec, split_k, stream);
        case 13:
            if (!vec) return launch_tile<128, 128, 4, 2, 4, 3, 2, 2>(p, vec, split_k, stream);
            return launch_tile<96, 128, 1, 4, 4, 3, 2, 2>(p, vec, split_k, stream);
        default: return launch_tile<256, 128, 4, 2, 4, 3, 2, 2>(p, vec, split_k, stream);
    }
}

}  // namespace conv
}  // namespace gpulet
