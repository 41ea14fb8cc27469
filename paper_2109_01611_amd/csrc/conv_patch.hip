// 3x3 convolutions of the forward pass served on a gpu-let (paper Sec. 5; the
// models of Table 4) that keep the input patch of a pixel tile in LDS instead of
// staging every pixel once per filter tap: the general kernel (any multiple of
// 64 input channels) and the variant for exactly 64 input channels whose
// weights stay in registers.
#include "conv_common.h"

namespace gpulet {
namespace conv {

namespace {

// ---------------------------------------------------------------------------
// 3x3 filters with stride 1 and C % 64 == 0: input patches stay in LDS.
//
// The implicit-GEMM A operand repeats every input pixel up to nine times, once
// per tap, and the kernel above stages all nine copies.  Here a workgroup
// stages, per block of 64 channels, the patch of input pixels its 128 output
// pixels touch (halo included) exactly once, and the nine taps read it at
// shifted positions.  Only the weights still move once per tap, three taps (one
// filter row) per ring step, so a step carries three times the arithmetic of a
// depth slice per workgroup barrier.
//
// Output pixels are ordered in column blocks of `tw` pixels: block cb holds
// columns cb*tw .. cb*tw+tw-1 of every output row, linearised as
// l = (n*P + p)*tw + tx; a tile is 128 consecutive l of one block.  With
// tw = Q this is the plain pixel order (tiles may cross rows and images); with
// tw = 16 a tile is an 8 x 16 pixel rectangle.  The patch is addressed by
// "virtual rows" v = n*(H+2) + h + pad, so the rows between two images are the
// zero padding, and holds rows v0 .. v0+prow-1, columns q0-pad .. q0+tw+pad-1
// of the block: position pos = (v - v0)*(tw+2) + u.  An output pixel with first
// virtual row v and block column tx reads tap (r, s) at
// pos = (v - v0 + r)*(tw+2) + tx + s = base + r*(tw+2) + s, base fixed per
// lane.  Each position is a 128-byte row of 64 channels whose 16-byte chunks are
// XOR-swizzled (patch_key) by q = pos - 2 * (patch row): along consecutive output
// pixels pos skips the two halo columns at the end of every block row, q does
// not, so any 16 consecutive pixels at one tap still cover all 64 LDS banks.
// (Swizzled by pos itself, every fragment read across such a seam cost an extra
// LDS cycle per 16 lanes.)  The host guarantees that no tile needs more than PMAX
// positions.
//
// Four consumer wavefronts (one per SIMD) own 32 tile rows x 64 channels each;
// four producers issue the transfers.  Patch buffers alternate per channel
// block, weight stages form a ring of three.  A producer's transfers complete
// in issue order, which the waits below rely on: within a step the pieces of
// the next patch are issued before the weights of step t+2, so waiting for the
// weights of step t also covers every patch piece issued earlier.
// ---------------------------------------------------------------------------
// STAMP: the instance that records wall-clock stamps of its first workgroups (gpulet_conv2d_timeline).
template <int BN, int NPROD, bool STAMP = false>
__global__ __launch_bounds__((4 + NPROD) * 64) void conv3x3_patch_kernel(const ConvParams p) {
    constexpr int BM = PATCH_BM, NCONS = 4, NS = 3, PMAX = PATCH_PMAX;
    constexpr int NT = BN / 32;                    // MFMA tiles per consumer (one row of them)
    constexpr int PATCH = PMAX * BK;               // elements per patch buffer
    constexpr int BSTAGE = 3 * BN * BK;            // elements per weight stage: the three taps of a filter row
    constexpr int POPS = PMAX / 8 / NPROD;         // patch transfers per producer lane and channel block
    constexpr int BOPS = 3 * BN / 8 / NPROD;       // weight transfers per producer lane and step
    constexpr int RG = BN / 8;                     // groups of 8 rows per weight tile
    static_assert(POPS % 2 == 0 && (3 * BN / 8) % NPROD == 0 && BN % 32 == 0, "transfer split");
    static_assert(POPS / 2 + 2 * BOPS <= 63, "6-bit transfer counter");
    constexpr int LDT = BN + 8;
    constexpr int MAIN = 2 * PATCH + NS * BSTAGE;
    constexpr int LDS_ELEMS = MAIN > BM * LDT * 2 ? MAIN : BM * LDT * 2;
    __shared__ __attribute__((aligned(1024))) __bf16 lds[LDS_ELEMS];
    // Per patch position: byte offset in x of its first channel (block 0), or OOB, with the
    // position's swizzle key in bits 4-6 (a pixel's channels start on a multiple of 128 bytes, so
    // the lane that fills physical chunk q gets its offset with one XOR by q << 4; an entry
    // with the OOB bit keeps it whatever is XORed or added below 2^31, and the hardware
    // answers such an offset with zeros).  Locating a position costs two divisions;
    // the 256 consumer threads compute one position each while the producers already fetch
    // weights, instead of every producer lane locating eight (which kept the first patch
    // transfer waiting for 0.9 us on a 10 us kernel).
    __shared__ unsigned ptab[PMAX];
    static_assert(PMAX == NCONS * 64, "one table entry per consumer thread");
    __bf16 *const patch = lds;
    __bf16 *const wring = lds + 2 * PATCH;

    long long t_start = 0;
    if constexpr (STAMP) t_start = wall_clock64();
    fetch_params(p);
    const int tile = tile_of_block(p);
    if (tile >= p.n_tiles) return;
    Stamps<STAMP> st(p, __builtin_amdgcn_readfirstlane(threadIdx.x >> 6));
    st.put(0, t_start);
    st.at(1);   // the argument block is there
    const int tm = fdiv(tile, p.d_tiles_n), tn = tile - tm * p.tiles_n;
    const int tl = fdiv(tm, p.d_ncb), cb = tm - tl * p.n_cb;
    const int l0 = tl * BM, n0 = tn * BN, q0 = cb * p.tw;
    // The bias is requested only once a wavefront's first transfers (or its table entry) are on
    // their way: a launch starts with cold instruction caches, and every instruction in front
    // of the first transfer delays it by its share of the fetch misses.
    BiasRegs bias_regs;
    const int NP = p.N * p.P;
    const int Hp = p.H + 2 * p.pad;       // virtual rows per image
    const int pwt = p.tw + 2;             // patch width: block columns plus the two halo columns
    const int nblk = p.C / BK;

    // Virtual row of output row rho at tap row 0.
    auto vrow = [&](int rho) {
        const int n = fdiv(rho, p.d_p);
        return n * Hp + (rho - n * p.P);
    };
    const int rho_first = fdiv(l0, p.d_tw);
    const int rho_last = min(NP - 1, fdiv(l0 + BM - 1, p.d_tw));
    const int v0 = vrow(rho_first);
    const int npos = (vrow(rho_last) + 2 - v0 + 1) * pwt;  // positions this tile needs (<= PMAX)

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    f32x16 acc[NT];  // consumers only

    if (wave >= NCONS) {
        // ------------------------------------------------------------ producer
        const int pw = wave - NCONS;
        const i32x4 rx = make_rsrc(p.x, p.x_bytes);
        const i32x4 rw = make_rsrc(p.w, p.w_bytes);

        // Weight transfer i fills rows rg*8 .. +8 of tap s of the stage, q = i*NPROD + pw = s*RG + rg.
        // NPROD divides RG, so s = (i*NPROD) / RG and rg = (i*NPROD) % RG + pw: the tap and the
        // row group's first part are known at compile time, and with NPROD even the chunk a lane
        // fills, (lane & 7) ^ ((row >> 1) & 7), is the same for every i.  One offset is computed
        // and the others follow by adding a constant times C (a few instructions in front of
        // the first transfer instead of a dozen per transfer).
        static_assert(RG % NPROD == 0 && NPROD % 2 == 0, "weight transfers: one chunk per lane");
        unsigned b_off[BOPS];
        {
            const int row0 = pw * 8 + (lane >> 3);
            const int cc = (lane & 7) ^ ((row0 >> 1) & 7);
            const unsigned first = static_cast<unsigned>((((n0 + row0) * 9) * p.C + cc * CHUNK) * 2);
            const int left = p.K - n0 - row0;   // rows from this lane's first one to the end of the filters
#pragma unroll
            for (int i = 0; i < BOPS; ++i) {
                const int s = (i * NPROD) / RG, rg = (i * NPROD) % RG;
                b_off[i] = rg * 8 < left ? first + static_cast<unsigned>((rg * 8 * 9 + s) * 2) * p.C : OOB;
            }
        }

        unsigned a_off[POPS];
        auto issue_patch = [&](int blk, int half) {
            const unsigned base = lds_addr(patch + (blk & 1) * PATCH) + pw * 1024;
            const unsigned add = static_cast<unsigned>(blk * BK * 2);
#pragma unroll
            for (int j = half * (POPS / 2); j < (half + 1) * (POPS / 2); ++j)
                dma16(rx, base + j * NPROD * 1024, blk < nblk ? a_off[j] + add : OOB);
        };
        // Weights of step t = 3*blk + r into ring stage `stage`.
        auto issue_weights = [&](int blk, int r, int stage) {
            const unsigned base = lds_addr(wring + stage * BSTAGE) + pw * 1024;
            const unsigned add = static_cast<unsigned>((r * 3 * p.C + blk * BK) * 2);
#pragma unroll
            for (int i = 0; i < BOPS; ++i) {
                dma16(rw, base + i * NPROD * 1024, blk < nblk ? b_off[i] + add : OOB);   // OOB + add stays out of bounds
            }
        };

        issue_weights(0, 0, 0);
        __syncthreads();   // the consumers have filled the position table
        // Patch transfer j of this wavefront fills positions (j*NPROD + pw)*8 .. +8;
        // this lane fills physical chunk lane&7 of one of them.
#pragma unroll
        for (int j = 0; j < POPS; ++j) a_off[j] = ptab[(j * NPROD + pw) * 8 + (lane >> 3)] ^ ((lane & 7u) << 4);
        issue_patch(0, 0);
        issue_patch(0, 1);
        bias_regs = load_bias<BN, (NCONS + NPROD) * 64>(p, n0);   // two plain loads: complete in order with the transfers
        issue_weights(0, 1, 1);   // not needed by the first step: behind the patch
        for (int blk = 0; blk < nblk; ++blk) {
            // step 3*blk: its weights were followed by those of step 3*blk+1 only
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(BOPS));
            __syncthreads();
            issue_patch(blk + 1, 0);
            issue_weights(blk, 2, 2);
            // step 3*blk+1: followed by half a patch and the weights of step 3*blk+2
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(POPS / 2 + BOPS));
            __syncthreads();
            issue_patch(blk + 1, 1);
            issue_weights(blk + 1, 0, 0);
            // step 3*blk+2: followed by the other half and the weights of step 3*blk+3
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(POPS / 2 + BOPS));
            __syncthreads();
            issue_weights(blk + 1, 1, 1);
        }
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    } else {
        // ------------------------------------------------------------ consumer
        const int frow = lane & 31, fhalf = lane >> 5;
        {
            // this thread's entry of the position table
            const int pos = wave * 64 + lane;
            const int vr = fdiv(pos, p.d_pwt), u = pos - vr * pwt;
            unsigned e = OOB;
            if (pos < npos) {
                const int v = v0 + vr;
                const int n = fdiv(v, p.d_hp);
                const int h = v - n * Hp - p.pad, w = q0 + u - p.pad;
                if (n < p.N && (unsigned)h < (unsigned)p.H && (unsigned)w < (unsigned)p.W)
                    e = static_cast<unsigned>((((n * p.H + h) * p.W + w) * p.C) * 2);
            }
            ptab[pos] = e | static_cast<unsigned>(patch_key(pos, vr) << 4);
        }
        __syncthreads();   // the table is complete (the producers wait here too)
        bias_regs = load_bias<BN, (NCONS + NPROD) * 64>(p, n0);
        st.at(2);
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

        // Patch position of this lane's tile row at tap (0, 0), and that position's patch row.
        int base = 0, brow = 0;
        {
            const int l = l0 + wave * 32 + frow;
            const int rho = fdiv(l, p.d_tw);
            if (rho < NP) {
                brow = vrow(rho) - v0;
                base = brow * pwt + (l - rho * p.tw);
            }
        }
        // A ring step is 12 depth steps of 16 (three taps x four).  The fragments of depth
        // step i+AHEAD are requested before the matrix instructions of step i are issued, so
        // LDS reads and matrix instructions overlap inside the one wavefront a SIMD runs.
        constexpr int KSTEPS = 3 * (BK / 16), AHEAD = 2;
        struct Frags {
            bf16x8 a, b[NT];
        };
        for (int blk = 0; blk < nblk; ++blk) {
            const __bf16 *pa = patch + (blk & 1) * PATCH;
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                __syncthreads();
                if (r == 0 && blk == 0) st.at(3);   // the first patch and weights have landed
                const __bf16 *wb = wring + r * BSTAGE;
                auto load = [&](Frags &f, int i) {
                    const int s = i / (BK / 16), ks = i % (BK / 16);
                    const int pos = base + r * pwt + s;
                    f.a = *reinterpret_cast<const bf16x8 *>(pa + pos * BK +
                                                            (((ks * 2 + fhalf) ^ patch_key(pos, brow + r)) * CHUNK));
#pragma unroll
                    for (int j = 0; j < NT; ++j)
                        f.b[j] = *reinterpret_cast<const bf16x8 *>(
                            &wb[s * BN * BK + lds_pos(j * 32 + frow, ks * 2 + fhalf)]);
                };
                Frags f[KSTEPS];
#pragma unroll
                for (int i = 0; i < AHEAD; ++i) load(f[i], i);
#pragma unroll
                for (int i = 0; i < KSTEPS; ++i) {
                    if (i + AHEAD < KSTEPS) load(f[i + AHEAD], i + AHEAD);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int j = 0; j < NT; ++j)
                        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i].a, f[i].b[j], acc[j], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    }

    // Epilogue through LDS, as in the kernel above.
    float *stg = reinterpret_cast<float *>(lds);
    st.at(4);          // end of the main loop
    __syncthreads();
    if (wave < NCONS) {
        const int frow = lane & 31, fhalf = lane >> 5;
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = wave * 32 + 8 * (v >> 2) + 4 * fhalf + (v & 3);
                stg[row * LDT + j * 32 + frow] = acc[j][v];
            }
    }
    __syncthreads();
    st.at(5);          // the tile is staged
    finish_tile<BM, BN, (NCONS + NPROD) * 64>(p, stg, n0, bias_regs, [&](int row) {
        const int l = l0 + row;
        const int rho = fdiv(l, p.d_tw);
        const int q = q0 + (l - rho * p.tw);
        return (rho < NP && q < p.Q) ? rho * p.Q + q : -1;
    });
    st.at(6);          // the output stores are issued
}

// ---------------------------------------------------------------------------
// 3x3 filters, stride 1, pad 1, exactly 64 input channels (the first stages of
// VGG-16 and ResNet-50): the weights stay in registers.
//
// With one block of 64 channels the patch kernel above would fetch all of a
// filter tile's weights (72 KB) for every 128 output pixels, more than the
// pixels themselves.  Here a workgroup owns one tile of 64 filters for its whole
// life and walks over many pixel tiles.  Its four consumer wavefronts are 2
// pixel halves x 2 filter halves (64 pixels x 32 filters each), and a consumer
// keeps the 36 fragments of its 32 filters (9 taps x 4 depth steps) in 144
// registers: in the main loop LDS serves only the input patch, two fragment
// reads for two matrix instructions.  Four producer wavefronts keep the patches
// of the next tiles in flight (two LDS buffers of 32 KB, DMA loads; a third buffer changed nothing).
//
// Per tile every wavefront executes two barriers:
//   B1(t): the patch of tile t has landed (each producer waited for its own
//          transfers; those of later tiles may still be in flight);
//   B2(t): the consumers have read the patch of tile t for the last time; the
//          producers refill that buffer with tile t+2.
// The product is taken as filters x pixels, so a lane ends up with groups of 4
// consecutive filters of one pixel; bias, ReLU and the rounding to bf16 happen
// in registers, and a piece of LDS private to the wavefront turns the groups
// into 16 bytes per lane with four consecutive lanes covering a pixel's 32
// filters (no workgroup barrier, 64-byte store segments).
// Taps and channels are summed in the order of the patch kernel and the bias
// is added last, so results are bit-identical to the other tiles.  No residual
// operand; K % 8 == 0 and a destination that allows aligned 16-byte stores.
// ---------------------------------------------------------------------------
// STAMP: the instance that records wall-clock stamps of its first workgroups (gpulet_conv2d_timeline):
// 0 first instruction, 1 weights requested, and for the workgroup's fourth pixel tile 2 before B1,
// 3 patch there (after B1), 4 matrix instructions issued, 5 patch released (after B2), 6 output
// stores issued, 7 the fifth tile before B1 (tile period = 7 - 2).
template <bool STAMP>
__global__ __launch_bounds__(512) void conv3x3_c64_kernel(const ConvParams p, const int wgs_per_col, const int tiles_m,
                                                          const int die_aware) {
    long long t_start = 0;
    if constexpr (STAMP) t_start = wall_clock64();
    fetch_params(p);
    asm volatile("" ::"s"(p.pool2));   // requested with the rest of the argument block
    constexpr int BM = PATCH_BM, BN = 64, NPROD = 4, PMAX = PATCH_PMAX, NB = 2;  // NB patch buffers
    constexpr int PATCH = PMAX * BK;           // elements per patch buffer
    constexpr int POPS = PMAX / 8 / NPROD;     // patch transfers per producer lane and tile
    constexpr int TROW = 32 * 2 + 16;          // bytes per pixel row of a consumer's transposition area (padded)
    static_assert(NB * POPS <= 63, "6-bit transfer counter");
    __shared__ __attribute__((aligned(1024))) __bf16 patch[NB * PATCH];
    __shared__ __attribute__((aligned(16))) unsigned char trs[4 * 64 * TROW];
    __shared__ __attribute__((aligned(16))) float lbias[BN];

    // Which pixel tiles this workgroup walks: first, stride, count (uniform over the workgroup).
    // Workgroups are dealt round-robin to the eight dies.  When the grid allows it every die
    // gets one contiguous eighth of the pixel tiles, which its workgroups (all filter tiles
    // included) sweep side by side: the halo rows and columns that neighbouring tiles share, and
    // the second read of a patch by the next filter tile, then hit that die's L2 instead of
    // crossing the fabric again.
    int col, first, step, T;
    if (die_aware) {
        const int die = blockIdx.x & 7, r = blockIdx.x >> 3;
        col = r % p.tiles_n;
        const int slot = r / p.tiles_n;
        const int per_die = (tiles_m + 7) >> 3;
        const int begin = die * per_die;
        const int count = min(per_die, tiles_m - begin);
        step = wgs_per_col >> 3;
        first = begin + slot;
        T = slot < count ? (count - slot + step - 1) / step : 0;
    } else {
        col = blockIdx.x % p.tiles_n;
        first = blockIdx.x / p.tiles_n;
        step = wgs_per_col;
        T = first < tiles_m ? (tiles_m - first + step - 1) / step : 0;
    }
    if (T <= 0) return;
    const int n0 = col * BN;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    Stamps<STAMP> st(p, wave);
    st.put(0, t_start);
    const int NP = p.N * p.P;
    const int Hp = p.H + 2 * p.pad;       // virtual rows per image
    const int pwt = p.tw + 2;             // patch width: block columns plus the two halo columns
    if (threadIdx.x < BN) {
        const int k = n0 + static_cast<int>(threadIdx.x);
        lbias[threadIdx.x] = (p.b && k < p.K) ? p.b[k] : 0.f;
    }

    auto vrow = [&](int rho) {
        const int n = fdiv(rho, p.d_p);
        return n * Hp + (rho - n * p.P);
    };
    // Pixel tile t of this workgroup: first linear pixel, first column, first virtual row.
    struct Tile {
        int l0, q0, v0, npos;
    };
    auto tile_at = [&](int t) {
        const int tm = first + t * step;
        const int tl = fdiv(tm, p.d_ncb), cb = tm - tl * p.n_cb;
        Tile r;
        r.l0 = tl * BM;
        r.q0 = cb * p.tw;
        const int rho_first = fdiv(r.l0, p.d_tw);
        const int rho_last = min(NP - 1, fdiv(r.l0 + BM - 1, p.d_tw));
        r.v0 = vrow(rho_first);
        r.npos = (vrow(rho_last) + 2 - r.v0 + 1) * pwt;  // positions this tile needs (<= PMAX)
        return r;
    };

    if (wave >= 4) {
        // ------------------------------------------------------------ producer
        const int pw = wave - 4;
        const i32x4 rx = make_rsrc(p.x, p.x_bytes);
        // Transfer j of this wavefront fills positions (j*NPROD + pw)*8 .. +8; this lane fills
        // physical chunk lane&7 of one of them.
        auto issue_patch = [&](int t) {
            const unsigned base = lds_addr(patch + (t % NB) * PATCH) + pw * 1024;
            Tile tl = tile_at(t < T ? t : 0);
            if (t >= T) tl.npos = 0;  // past the end: the transfers still run (fixed count) and write zeros
#pragma unroll
            for (int j = 0; j < POPS; ++j) {
                const int pos = (j * NPROD + pw) * 8 + (lane >> 3);
                const int vr = fdiv(pos, p.d_pwt), u = pos - vr * pwt;
                const int cc = (lane & 7) ^ patch_key(pos, vr);
                unsigned off = OOB;
                if (pos < tl.npos) {
                    const int v = tl.v0 + vr;
                    const int n = fdiv(v, p.d_hp);
                    const int h = v - n * Hp - p.pad, w = tl.q0 + u - p.pad;
                    if (n < p.N && (unsigned)h < (unsigned)p.H && (unsigned)w < (unsigned)p.W)
                        off = static_cast<unsigned>((((n * p.H + h) * p.W + w) * BK + cc * CHUNK) * 2);
                }
                dma16(rx, base + j * NPROD * 1024, off);
            }
        };
#pragma unroll
        for (int t = 0; t < NB; ++t) issue_patch(t);
        for (int t = 0; t < T; ++t) {
            __builtin_amdgcn_s_waitcnt(vmcnt_imm((NB - 1) * POPS));  // all but the transfers of later tiles have landed
            __syncthreads();                                         // B1
            __syncthreads();                                         // B2
            issue_patch(t + NB);
        }
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    } else {
        // ------------------------------------------------------------ consumer
        const int frow = lane & 31, fhalf = lane >> 5;
        const int wy = wave >> 1, wx = wave & 1;   // pixel half, filter half
        // The fragments of this wavefront's 32 filters: tap-major, four depth steps of 16 each.
        bf16x8 wf[36];
        {
            const __amdgpu_buffer_rsrc_t rw =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<__bf16 *>(p.w), 0, p.w_bytes, RSRC_FLAGS);
            const int k = n0 + wx * 32 + frow;
#pragma unroll
            for (int i = 0; i < 36; ++i) {
                const int tap = i >> 2, ks = i & 3;
                const unsigned off = k < p.K ? static_cast<unsigned>(((k * 9 + tap) * BK + (ks * 2 + fhalf) * CHUNK) * 2) : OOB;
                const u32x4 raw = __builtin_amdgcn_raw_buffer_load_b128(rw, off, 0, 0);
                wf[i] = __builtin_bit_cast(bf16x8, raw);
            }
        }
        st.at(1);
        unsigned char *tr = trs + wave * (64 * TROW);
        const unsigned limit = relu_limit(p.relu);
        const int kst = n0 + wx * 32 + (lane & 3) * 8;   // first of the 8 filters this lane stores

        for (int t = 0; t < T; ++t) {
            const Tile tl = tile_at(t);
            // Patch positions of this lane's two pixels at tap (0, 0).
            int base[2], brow[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int l = tl.l0 + wy * 64 + i * 32 + frow;
                const int rho = fdiv(l, p.d_tw);
                brow[i] = rho < NP ? vrow(rho) - tl.v0 : 0;
                base[i] = rho < NP ? brow[i] * pwt + (l - rho * p.tw) : 0;
            }
            f32x16 acc[2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
            if (t == 3) st.at(2);
            if (t == 4) st.at(7);
            __syncthreads();  // B1
            if (t == 3) st.at(3);
            const __bf16 *pa = patch + (t % NB) * PATCH;
            // The fragments of depth step i+AHEAD are requested before the matrix instructions of
            // step i are issued, so LDS reads and matrix instructions overlap inside the wavefront.
            constexpr int AHEAD = 2;
            struct Frags {
                bf16x8 a[2];
            };
            auto load = [&](Frags &f, int i) {
                const int tap = i >> 2, ks = i & 3;
                const int r = tap / 3, sx = tap - r * 3;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int pos = base[h] + r * pwt + sx;
                    f.a[h] = *reinterpret_cast<const bf16x8 *>(pa + pos * BK + (((ks * 2 + fhalf) ^ patch_key(pos, brow[h] + r)) * CHUNK));
                }
            };
            Frags f[36];
#pragma unroll
            for (int i = 0; i < AHEAD; ++i) load(f[i], i);
#pragma unroll
            for (int i = 0; i < 36; ++i) {
                if (i + AHEAD < 36) load(f[i + AHEAD], i + AHEAD);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    acc[h] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i], f[i].a[h], acc[h], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (t == 3) st.at(4);
            __syncthreads();  // B2
            if (t == 3) st.at(5);

            // Register v of a lane: filter 8*(v/4) + 4*(lane/32) + v%4 of the 32, pixel lane%32 (+32 h).
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 b4 = *reinterpret_cast<const float4 *>(&lbias[wx * 32 + 8 * g + 4 * fhalf]);
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    *reinterpret_cast<uint2 *>(tr + (h * 32 + frow) * TROW + g * 16 + fhalf * 8) = make_uint2(
                        relu_or_pass(pack_bf16(acc[h][4 * g] + b4.x, acc[h][4 * g + 1] + b4.y), limit),
                        relu_or_pass(pack_bf16(acc[h][4 * g + 2] + b4.z, acc[h][4 * g + 3] + b4.w), limit));
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            if (p.pool2) {
                // A 2x2 / stride 2 max pool follows: the wavefront's 64 pixels are 64/tw whole rows of
                // the tile (an even number, starting at an even row and column), i.e. 16 windows;
                // lane -> window lane/4, its 8 filters.  The maximum is taken on the rounded values,
                // as the pool kernel would, and only the pooled pixel is stored.  p.th = log2(tw/2).
                const int pp = lane >> 2, py = pp >> p.th, px = pp - (py << p.th);
                const int lw = 2 * py * p.tw + 2 * px;            // window's top left pixel among the 64
                unsigned k[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint4 v = *reinterpret_cast<const uint4 *>(tr + (lw + (i >> 1) * p.tw + (i & 1)) * TROW + (lane & 3) * 16);
                    const unsigned kv[4] = {bf16_pair_order_key(v.x), bf16_pair_order_key(v.y), bf16_pair_order_key(v.z),
                                            bf16_pair_order_key(v.w)};
#pragma unroll
                    for (int e = 0; e < 4; ++e) k[e] = i == 0 ? kv[e] : max_keys(k[e], kv[e]);
                }
                const int l = tl.l0 + wy * 64 + lw;
                const int rho = fdiv(l, p.d_tw);
                const int q = tl.q0 + (l - rho * p.tw);
                if (rho < NP && q < p.Q && kst < p.K)   // rho = n*P + row with P even: the pooled row is rho/2
                    *reinterpret_cast<uint4 *>(p.y + (((rho >> 1) * (p.Q >> 1) + (q >> 1)) * p.ldy + p.y_off + kst)) =
                        make_uint4(bf16_pair_order_key(k[0]), bf16_pair_order_key(k[1]), bf16_pair_order_key(k[2]),
                                   bf16_pair_order_key(k[3]));
            } else {
            uint4 out[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                out[i] = *reinterpret_cast<const uint4 *>(tr + ((lane >> 2) + i * 16) * TROW + (lane & 3) * 16);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int l = tl.l0 + wy * 64 + (lane >> 2) + i * 16;
                const int rho = fdiv(l, p.d_tw);
                const int q = tl.q0 + (l - rho * p.tw);
                if (rho < NP && q < p.Q && kst < p.K)
                    *reinterpret_cast<uint4 *>(p.y + ((rho * p.Q + q) * p.ldy + p.y_off + kst)) = out[i];
            }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            if (t == 3) st.at(6);
        }
    }
}

// Column-block width for the patch kernel and whether every tile's patch fits PATCH_PMAX
// positions.  Small images use the whole row (tiles then cross rows and images), wide ones
// 16-pixel blocks (tiles are 8 x 16 rectangles) or 14-pixel blocks when that divides the row.
bool patch_geometry(const ConvParams &p, int *tw_out) {
    int tw;
    if (p.Q <= 16) tw = p.Q;
    else if (p.Q % 16 == 0) tw = 16;
    else if (p.Q % 14 == 0) tw = 14;
    else tw = 16;
    const int NP = p.N * p.P, Hp = p.H + 2 * p.pad;
    const long long lin = 1LL * NP * tw;
    int worst = 0;
    for (long long l0 = 0; l0 < lin; l0 += PATCH_BM) {
        const int r0 = static_cast<int>(l0 / tw);
        const int r1 = static_cast<int>(std::min<long long>(NP - 1, (l0 + PATCH_BM - 1) / tw));
        const int v0 = (r0 / p.P) * Hp + r0 % p.P, v1 = (r1 / p.P) * Hp + r1 % p.P + 2;
        worst = std::max(worst, (v1 - v0 + 1) * (tw + 2));
        if (worst > PATCH_PMAX) return false;
    }
    *tw_out = tw;
    return true;
}

}  // namespace

bool patch_eligible(const ConvParams &p, bool vec, int *tw_out) {
    return vec && p.ldx == p.C && p.R == 3 && p.S == 3 && p.stride == 1 && p.pad == 1 && p.C % BK == 0 && p.P == p.H &&
           p.Q == p.W && patch_geometry(p, tw_out);
}

hipError_t launch_patch(ConvParams p, int tw, hipStream_t stream) {
    constexpr int BN = 64;
    p.tw = tw;
    p.n_cb = (p.Q + tw - 1) / tw;
    const long long lin = 1LL * p.N * p.P * tw;
    const int tiles_m = static_cast<int>((lin + PATCH_BM - 1) / PATCH_BM) * p.n_cb;
    p.tiles_n = (p.K + BN - 1) / BN;
    p.n_tiles = tiles_m * p.tiles_n;
    p.split_k = 1;
    p.tiles_per_xcd = (p.n_tiles + 7) / 8;
    p.d_tiles_n = make_fastdiv(p.tiles_n);
    p.d_tw = make_fastdiv(tw);
    p.d_ncb = make_fastdiv(p.n_cb);
    p.d_pwt = make_fastdiv(tw + 2);
    p.d_hp = make_fastdiv(p.H + 2 * p.pad);
    if (p.stamps)
        hipLaunchKernelGGL((conv3x3_patch_kernel<BN, 4, true>), dim3(static_cast<unsigned>(p.tiles_per_xcd * 8)),
                           dim3(8 * 64), 0, stream, p);
    else
        hipLaunchKernelGGL((conv3x3_patch_kernel<BN, 4>), dim3(static_cast<unsigned>(p.tiles_per_xcd * 8)),
                           dim3(8 * 64), 0, stream, p);
    return hipGetLastError();
}

// The 3x3 kernel with register-resident weights: what the patch kernel needs, exactly 64 input
// channels, no residual operand, aligned 16-byte stores.
bool c64_applicable(const ConvParams &p, bool vec, int *tw_out, bool pool2) {
    if (!(patch_eligible(p, vec, tw_out) && p.C == BK && !p.res && p.vec_store && p.K % 8 == 0)) return false;
    // a fused 2x2 pool: every wavefront's 64 pixels must be an even number of whole, even-aligned tile rows
    const int tw = *tw_out;
    return !pool2 || (p.relu && p.P % 2 == 0 && p.Q % 2 == 0 && tw >= 2 && tw <= 32 && (tw & (tw - 1)) == 0);
}

hipError_t launch_c64(ConvParams p, int tw, int n_cu, bool pool2, hipStream_t stream) {
    p.pool2 = pool2 ? 2 : 0;
    p.th = 0;
    while (pool2 && (2 << p.th) < tw) ++p.th;   // log2(tw / 2)
    p.tw = tw;
    p.n_cb = (p.Q + tw - 1) / tw;
    const long long lin = 1LL * p.N * p.P * tw;
    const int tiles_m = static_cast<int>((lin + PATCH_BM - 1) / PATCH_BM) * p.n_cb;
    p.tiles_n = (p.K + 63) / 64;
    p.n_tiles = tiles_m * p.tiles_n;
    p.split_k = 1;
    p.d_tw = make_fastdiv(tw);
    p.d_ncb = make_fastdiv(p.n_cb);
    p.d_pwt = make_fastdiv(tw + 2);
    p.d_hp = make_fastdiv(p.H + 2 * p.pad);
    // one workgroup per CU (registers), all resident at once; a multiple of 8 per filter tile
    // where possible, so that every die can own a contiguous eighth of the pixel tiles
    int wgs_per_col = std::max(1, std::min(tiles_m, n_cu / p.tiles_n));
    const int die_aware = wgs_per_col >= 8 ? 1 : 0;
    if (die_aware) wgs_per_col &= ~7;
    if (p.stamps)
        hipLaunchKernelGGL(conv3x3_c64_kernel<true>, dim3(static_cast<unsigned>(wgs_per_col * p.tiles_n)), dim3(512), 0, stream, p,
                           wgs_per_col, tiles_m, die_aware);
    else
        hipLaunchKernelGGL(conv3x3_c64_kernel<false>, dim3(static_cast<unsigned>(wgs_per_col * p.tiles_n)), dim3(512), 0, stream, p,
                           wgs_per_col, tiles_m, die_aware);
    return hipGetLastError();
}

}  // namespace conv
}  // namespace gpulet
