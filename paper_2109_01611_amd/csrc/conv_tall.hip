// 3x3 convolutions of the forward pass served on a gpu-let (paper Sec. 5; the
// models of Table 4) on layers with many output tiles: a tall pixel tile whose
// input patch stays in LDS, weights streamed one filter tap at a time.
#include "conv_common.h"

namespace gpulet {
namespace conv {

namespace {

// ---------------------------------------------------------------------------
// 3x3 filters, stride 1, pad 1, C % 64 == 0, dense input pixels.
//
// What bounds the other kernels on large layers is the traffic through LDS: the
// gathering kernel stages every input pixel once per filter tap, the 128 x 64
// patch kernel re-reads a weight fragment for every 32 pixels.  Here a
// workgroup owns a th x tw rectangle of one image's output pixels with
// th * tw <= 224 (seven matrix-instruction row tiles; 8 x 28 on the 56, 112 and
// 224 pixel wide maps of the served models) and 128 filters:
//
//   * per block of 64 channels the (th+2) x (tw+2) input patch is staged once
//     (two buffers, the next block's patch arrives during the first five taps);
//   * the weights of one tap (128 filters x 64 channels, 16 KB) form a ring
//     step; four stages, so that two steps are in flight while the step being
//     multiplied and the one after it have landed;
//   * eight consumer wavefronts = four groups of 32 filters x two sets of row
//     tiles (four and three).  Wavefront w runs on SIMD w % 4, so every SIMD
//     hosts a four-tile and a three-tile consumer of the same filters: seven
//     row tiles per SIMD, each weight fragment read serves four (three) matrix
//     instructions.  That is 9 fragment reads per 7 matrix instructions against
//     12 per 8 in the 128 x 64 patch kernel, and 178 KB staged per 33 MFLOP.
//
// A patch position is a 128-byte row of 64 channels.  Output pixel l = ty*tw + tx
// of the tile reads tap (r, s) at position (ty + r)*(tw + 2) + tx + s: along a
// fragment's 32 consecutive pixels the position steps by one, except from the end
// of a tile row to the start of the next, where it skips the two halo columns.
// The 16-byte chunks of a position are therefore XOR-swizzled not by the position
// but by q = position - 2 * (patch row) = l + r*tw + s, which steps by one over
// that seam too: any 16 consecutive pixels at one tap then cover all 64 banks
// (the skip is odd, so even and odd positions still alternate, and each parity
// sees eight consecutive values of q >> 1).  Swizzled by position, every fragment
// read that spans a seam took an extra LDS cycle per 16 lanes (6.4 instead of 4
// cycles per read, measured with the bank-conflict counter).
//
// Synchronisation: one workgroup barrier per tap.  Barrier g means: the weights
// of taps <= g+1 (and the patch of the block tap g+1 belongs to) have landed,
// and every consumer has finished reading tap g-1, whose stage the producers
// refill with tap g+3.  Because the data of tap g+1 is already there, a
// consumer requests the first fragments of the next tap before it reaches the
// next barrier: the barrier is flow control only, and no wavefront waits for
// LDS behind it.  A producer's transfers complete in issue order, so "tap g+1
// has landed" is a bound on its outstanding transfers.
//
// Channels are summed in blocks of 64 with the taps inside a block, as in the
// gathering kernel's tap-inner order and the patch kernel: results are
// bit-identical to those.
// ---------------------------------------------------------------------------
constexpr int TALL_BM = 224;     // tile rows = 7 matrix-instruction row tiles
constexpr int TALL_BN = 128;
constexpr int TALL_PMAX = 320;   // patch positions per buffer (40 KB)

struct TallFrags {
    bf16x8 a[4], b;
};

// LDS byte offset -> fragment.  `lds` is the kernel's __shared__ array, so the compiler emits
// a ds_read_b128 with the offset as its address.
__device__ __forceinline__ bf16x8 lds_frag(const __bf16 *lds, unsigned byte_off) {
    return *reinterpret_cast<const bf16x8 *>(reinterpret_cast<const char *>(lds) + byte_off);
}

// One consumer wavefront: MTW row tiles starting at row tile rt0, filters fg*32 .. +32.
// a_addr[i][tap]: byte offset of this lane's fragment of depth step 0 at tap `tap` for its row
// of row tile i, inside patch buffer 0; depth step ks is at a_addr ^ (ks << 5).
template <int MTW, bool STAMP>
__device__ __forceinline__ void tall_consume(const __bf16 *lds, const unsigned (&a_addr)[4][9], const unsigned b_addr,
                                             const int nblk, const unsigned wring_off, const unsigned stage_bytes,
                                             const unsigned patch_bytes, f32x16 (&acc)[4], Stamps<STAMP> &st) {
    TallFrags f0, f1;
    // Zero, but re-made opaque to the compiler in every block: the offsets of the four depth
    // steps of every (row tile, tap) are loop invariants, and hoisting them out of the block
    // loop would cost 150 registers.  Kept variable, a fragment address is one xor-add.
    unsigned zero = 0;
    // Fragments of depth step ks of tap `tap`: patch buffer offset pb, weight stage offset st.
    auto load = [&](TallFrags &f, int tap, int ks, unsigned pb, unsigned st) {
        const unsigned kx = static_cast<unsigned>(ks << 5) | zero;
        f.b = lds_frag(lds, (b_addr ^ kx) + st);
#pragma unroll
        for (int i = 0; i < MTW; ++i) f.a[i] = lds_frag(lds, (a_addr[i][tap] ^ kx) + pb);
    };
    auto mma = [&](const TallFrags &f) {
#pragma unroll
        for (int i = 0; i < MTW; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b, acc[i], 0, 0, 0);
    };
    unsigned pb = 0;                       // byte offset of the current block's patch buffer
    int g = 0;                             // tap counter over all blocks: its weights sit in stage g % 4
    __syncthreads();                       // barrier 0
    st.at(3);                              // the first patch and weights have landed
    load(f0, 0, 0, 0u, wring_off);
    for (int blk = 0; blk < nblk; ++blk) {
        const unsigned pb_next = pb ^ patch_bytes;   // pb is only ever 0 or patch_bytes
        asm volatile("" : "+s"(zero));
#pragma unroll
        for (int tap = 0; tap < 9; ++tap, ++g) {
            const unsigned st = wring_off + static_cast<unsigned>(g & 3) * stage_bytes;
            const unsigned st_next = wring_off + static_cast<unsigned>((g + 1) & 3) * stage_bytes;
            if (g > 0) __syncthreads();    // barrier g
            // four depth steps of 16; the fragments of the next step are requested before this
            // step's matrix instructions are issued
            load(f1, tap, 1, pb, st);
            __builtin_amdgcn_sched_barrier(0);
            mma(f0);
            __builtin_amdgcn_sched_barrier(0);
            load(f0, tap, 2, pb, st);
            __builtin_amdgcn_sched_barrier(0);
            mma(f1);
            __builtin_amdgcn_sched_barrier(0);
            load(f1, tap, 3, pb, st);
            __builtin_amdgcn_sched_barrier(0);
            mma(f0);
            __builtin_amdgcn_sched_barrier(0);
            // first step of the next tap: its weights landed before barrier g; past the last
            // tap this reads a stage nobody uses (the values are dropped)
            if (tap < 8)
                load(f0, tap + 1, 0, pb, st_next);
            else
                load(f0, 0, 0, pb_next, st_next);
            __builtin_amdgcn_sched_barrier(0);
            mma(f1);
            __builtin_amdgcn_sched_barrier(0);
        }
        pb = pb_next;
    }
}

// Epilogue of a tile whose layer is followed by a 2x2 / stride 2 max pool: the fp32 tile parked in
// LDS (rows = the th x tw pixels of the tile, th, tw and the tile's origin even) is reduced over
// each 2x2 window, then bias, ReLU and the rounding to bf16 are applied once and only the pooled
// pixel is stored.  x -> round(relu(x + bias)) does not decrease, so the maximum can be taken
// first: the bits equal those of the layer's output pooled by the pool kernel.
template <int BN, int NTHR>
__device__ __forceinline__ void finish_tile_pool2(const ConvParams &p, const float *stg, int n0, const BiasRegs &br,
                                                  int n, int ty0, int tx0) {
    constexpr int LDT = BN + 8, VPR = BN / 8, PSTEP = NTHR / VPR;
    const int cv = threadIdx.x % VPR, k = n0 + cv * 8;
    if (k >= p.K) return;
    const float bias[8] = {br.lo.x, br.lo.y, br.lo.z, br.lo.w, br.hi.x, br.hi.y, br.hi.z, br.hi.w};
    const unsigned limit = relu_limit(p.relu);
    const int tw2 = p.tw >> 1, n_pooled = (p.th >> 1) * tw2;
    const int P2 = p.P >> 1, Q2 = p.Q >> 1;
    __bf16 *yb = p.y + p.y_off + k;
    for (int pi = threadIdx.x / VPR; pi < n_pooled; pi += PSTEP) {
        const int py = pi / tw2, px = pi - py * tw2;
        const int hh = ty0 + 2 * py, ww = tx0 + 2 * px;     // top left pixel of the window
        if (hh >= p.P || ww >= p.Q) continue;               // P, Q, hh, ww even: the window is inside or outside as a whole
        const int row = 2 * py * p.tw + 2 * px;
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = -__builtin_inff();
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const float *src = &stg[(row + (t >> 1) * p.tw + (t & 1)) * LDT + cv * 8];
            const float4 lo = *reinterpret_cast<const float4 *>(src);
            const float4 hi = *reinterpret_cast<const float4 *>(src + 4);
            const float u[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = u[e] > v[e] ? u[e] : v[e];
        }
        unsigned pk[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            pk[e] = relu_or_pass(pack_bf16(v[2 * e] + bias[2 * e], v[2 * e + 1] + bias[2 * e + 1]), limit);
        const int m = (n * P2 + (hh >> 1)) * Q2 + (ww >> 1);
        *reinterpret_cast<uint4 *>(yb + m * p.ldy) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
    }
}

// STAMP: the instance that records wall-clock stamps of its first workgroups (gpulet_conv2d_timeline).
template <bool STAMP>
__global__ __launch_bounds__(768) void conv3x3_tall_kernel(const ConvParams p) {
    constexpr int BM = TALL_BM, BN = TALL_BN, NCONS = 8, NPROD = 4, NS = 4, PMAX = TALL_PMAX;
    constexpr int WSTAGE = BN * BK;                // elements per weight stage: one tap
    constexpr int PATCH = PMAX * BK;               // elements per patch buffer
    constexpr int POPS = PMAX / 8 / NPROD;         // patch transfers per producer lane and channel block
    constexpr int WOPS = BN / 8 / NPROD;           // weight transfers per producer lane and tap
    constexpr int PP_TAPS = 5, PP_PER = POPS / PP_TAPS;   // the next patch is issued over the first taps of a block
    static_assert(POPS % PP_TAPS == 0 && WOPS + PP_PER <= 63, "transfer split / 6-bit transfer counter");
    constexpr int LDT = BN + 8;
    constexpr int MAIN = NS * WSTAGE + 2 * PATCH;
    constexpr int LDS_ELEMS = MAIN > BM * LDT * 2 ? MAIN : BM * LDT * 2;
    __shared__ __attribute__((aligned(1024))) __bf16 lds[LDS_ELEMS];
    // Per patch position: byte offset in x of its first channel (block 0), or OOB, with the
    // position's swizzle key in bits 4-6 (as in the patch kernel: one XOR by the lane's chunk
    // gives its offset, and the OOB bit survives it); filled by the consumer threads (one
    // position each) while the producers already fetch weights.
    __shared__ unsigned ptab[PMAX];
    static_assert(PMAX <= NCONS * 64, "one table entry per consumer thread");
    __bf16 *const wring = lds;
    __bf16 *const patch = lds + NS * WSTAGE;

    long long t_start = 0;
    if constexpr (STAMP) t_start = wall_clock64();
    fetch_params(p);
    asm volatile("" ::"s"(p.pool2));   // requested with the rest of the argument block
    const int tile = tile_of_block(p);
    if (tile >= p.n_tiles) return;
    Stamps<STAMP> st(p, __builtin_amdgcn_readfirstlane(threadIdx.x >> 6));
    st.put(0, t_start);
    st.at(1);   // the argument block is there
    // tile -> (image, tile row, tile column, filter tile); filter tiles of one pixel tile are neighbours
    const int tm = fdiv(tile, p.d_tiles_n), tn = tile - tm * p.tiles_n;
    const int n = fdiv(tm, p.d_hp), ti = tm - n * p.tiles_img;
    const int tyi = fdiv(ti, p.d_ncb), txi = ti - tyi * p.n_cb;
    const int ty0 = tyi * p.th, tx0 = txi * p.tw, n0 = tn * BN;
    BiasRegs bias_regs;   // requested once a wavefront's first transfers (or its table entry) are on their way
    const int pwt = p.tw + 2;                      // patch width: tile columns plus the two halo columns
    const int npix = p.th * p.tw;                  // tile rows that are pixels
    const int npos = (p.th + 2) * pwt;             // patch positions in use (<= PMAX)
    const int nblk = p.C / BK;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    f32x16 acc[4];  // consumers only

    if (wave >= NCONS) {
        // ------------------------------------------------------------ producer
        const int pw = wave - NCONS;
        const i32x4 rx = make_rsrc(p.x, p.x_bytes);
        const i32x4 rw = make_rsrc(p.w, p.w_bytes);

        unsigned a_off[POPS];
        // Weight transfer i fills rows (i*NPROD + pw)*8 .. +8 of the stage.
        // Rows i*NPROD*8 further down change nothing in the chunk a lane fills (NPROD * 4 is a
        // multiple of 8): one offset is computed, the others add a constant times C.
        static_assert((NPROD * 4) % 8 == 0, "weight transfers: one chunk per lane");
        unsigned b_off[WOPS];
        {
            const int row0 = pw * 8 + (lane >> 3);
            const int cc = (lane & 7) ^ ((row0 >> 1) & 7);
            const unsigned first = static_cast<unsigned>((((n0 + row0) * 9) * p.C + cc * CHUNK) * 2);
            const int left = p.K - n0 - row0;   // rows from this lane's first one to the end of the filters
#pragma unroll
            for (int i = 0; i < WOPS; ++i)
                b_off[i] = i * NPROD * 8 < left ? first + static_cast<unsigned>(i * NPROD * 8 * 9 * 2) * p.C : OOB;
        }

        // Pieces first .. first+count-1 of the patch of channel block blk.
        auto issue_patch = [&](int blk, int first, int count) {
            const unsigned base = lds_addr(patch + (blk & 1) * PATCH) + pw * 1024;
            const unsigned add = static_cast<unsigned>(blk * BK * 2);
#pragma unroll
            for (int j = first; j < first + count; ++j) {
                dma16(rx, base + j * NPROD * 1024, blk < nblk ? a_off[j] + add : OOB);   // OOB + add stays out of bounds
            }
        };
        // Weights of tap `tap` of block blk, tap counter g, into stage g % NS.
        auto issue_weights = [&](int blk, int tap, int g) {
            const unsigned base = lds_addr(wring + (g & (NS - 1)) * WSTAGE) + pw * 1024;
            const unsigned add = static_cast<unsigned>((tap * p.C + blk * BK) * 2);
#pragma unroll
            for (int i = 0; i < WOPS; ++i) {
                dma16(rw, base + i * NPROD * 1024, blk < nblk ? b_off[i] + add : OOB);
            }
        };

        issue_weights(0, 0, 0);
        issue_weights(0, 1, 1);
        __syncthreads();   // the consumers have filled the position table
        // Patch transfer j of this wavefront fills positions (j*NPROD + pw)*8 .. +8; this lane
        // fills physical chunk lane&7 of one of them.
#pragma unroll
        for (int j = 0; j < POPS; ++j) a_off[j] = ptab[(j * NPROD + pw) * 8 + (lane >> 3)] ^ ((lane & 7u) << 4);
        issue_patch(0, 0, POPS);
        bias_regs = load_bias<BN, (NCONS + NPROD) * 64>(p, n0);   // plain loads complete in order with the transfers
        issue_weights(0, 2, 2);
        int g = 0;
        for (int blk = 0; blk < nblk; ++blk) {
#pragma unroll
            for (int tap = 0; tap < 9; ++tap, ++g) {
                // Tap g+1 has landed: behind it in issue order are only the patch pieces of the
                // previous step (taps 1..5 follow a step that issued some) and the weights of tap g+2.
                if (tap >= 1 && tap <= PP_TAPS)
                    __builtin_amdgcn_s_waitcnt(vmcnt_imm(WOPS + PP_PER));
                else
                    __builtin_amdgcn_s_waitcnt(vmcnt_imm(WOPS));
                __syncthreads();           // barrier g
                if (tap < PP_TAPS) issue_patch(blk + 1, tap * PP_PER, PP_PER);
                if (tap + 3 < 9)
                    issue_weights(blk, tap + 3, g + 3);
                else
                    issue_weights(blk + 1, tap + 3 - 9, g + 3);
            }
        }
        // Every transfer has landed before the epilogue reuses the memory.
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    } else {
        // ------------------------------------------------------------ consumer
        const int frow = lane & 31, fhalf = lane >> 5;
        const int fg = wave & 3, hi = wave >> 2;   // filter group; row tiles 0..3 or 4..6
        const int rt0 = hi * 4;
        {
            // this thread's entry of the position table
            const int pos = wave * 64 + lane;
            if (pos < PMAX) {
                const int vr = fdiv(pos, p.d_pwt), u = pos - vr * pwt;
                unsigned e = OOB;
                if (pos < npos) {
                    const int h = ty0 + vr - 1, w = tx0 + u - 1;
                    if ((unsigned)h < (unsigned)p.H && (unsigned)w < (unsigned)p.W)
                        e = static_cast<unsigned>((((n * p.H + h) * p.W + w) * p.C) * 2);
                }
                ptab[pos] = e | static_cast<unsigned>(patch_key(pos, vr) << 4);
            }
        }
        __syncthreads();   // the table is complete (the producers wait here too)
        st.at(2);
        bias_regs = load_bias<BN, (NCONS + NPROD) * 64>(p, n0);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
        unsigned a_addr[4][9];
        const unsigned patch0 = static_cast<unsigned>(NS * WSTAGE * 2);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int l = (rt0 + i) * 32 + frow;
            if (l >= npix) l = 0;                  // rows past the tile read pixel 0; their results are dropped
            const int ty = fdiv(l, p.d_tw), tx = l - ty * p.tw;
            const int base = ty * pwt + tx;
#pragma unroll
            for (int tap = 0; tap < 9; ++tap) {
                const int pos = base + (tap / 3) * pwt + (tap % 3);
                const int q = l + (tap / 3) * p.tw + (tap % 3);     // = pos - 2 * (patch row of pos)
                a_addr[i][tap] = patch0 + static_cast<unsigned>(pos * (BK * 2) + ((((q >> 1) & 7) ^ fhalf) << 4));
            }
        }
        const int brow = fg * 32 + frow;
        const unsigned b_addr = static_cast<unsigned>(brow * (BK * 2) + ((((brow >> 1) & 7) ^ fhalf) << 4));
        if (hi == 0)
            tall_consume<4, STAMP>(lds, a_addr, b_addr, nblk, 0u, WSTAGE * 2, PATCH * 2, acc, st);
        else
            tall_consume<3, STAMP>(lds, a_addr, b_addr, nblk, 0u, WSTAGE * 2, PATCH * 2, acc, st);
    }

    // Epilogue through LDS, as in the other kernels.
    float *stg = reinterpret_cast<float *>(lds);
    st.at(4);          // end of the main loop
    __syncthreads();   // all LDS reads of the main loop are done, all transfers have landed
    if (wave < NCONS) {
        const int frow = lane & 31, fhalf = lane >> 5;
        const int fg = wave & 3, hi = wave >> 2;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (hi * 4 + i >= BM / 32) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = (hi * 4 + i) * 32 + 8 * (v >> 2) + 4 * fhalf + (v & 3);
                stg[row * LDT + fg * 32 + frow] = acc[i][v];
            }
        }
    }
    __syncthreads();
    st.at(5);          // the tile is staged
    if (p.pool2) {
        finish_tile_pool2<BN, (NCONS + NPROD) * 64>(p, stg, n0, bias_regs, n, ty0, tx0);
    } else {
        finish_tile<BM, BN, (NCONS + NPROD) * 64>(p, stg, n0, bias_regs, [&](int row) {
            if (row >= npix) return -1;
            const int ty = fdiv(row, p.d_tw), tx = row - ty * p.tw;
            const int hh = ty0 + ty, ww = tx0 + tx;
            return (hh < p.P && ww < p.Q) ? (n * p.P + hh) * p.Q + ww : -1;
        });
    }
    st.at(6);          // the output stores are issued
}

// The pixel rectangle th x tw (th*tw <= 224, patch within TALL_PMAX positions) that wastes the
// fewest tile rows on a P x Q map; on a tie the wider one (longer contiguous runs per transfer).
bool tall_geometry(int P, int Q, bool even, int *th_out, int *tw_out, double *eff_out) {
    double best = 0.0;
    int bth = 0, btw = 0;
    const int step = even ? 2 : 1;     // tiles of whole 2x2 windows for a fused pool
    for (int tw = step; tw <= std::min(Q, TALL_BM); tw += step) {
        const int th_max = std::min(P, TALL_BM / tw);
        for (int th = step; th <= th_max; th += step) {
            if ((th + 2) * (tw + 2) > TALL_PMAX) break;
            const long long tiles = 1LL * ((P + th - 1) / th) * ((Q + tw - 1) / tw);
            const double eff = static_cast<double>(P) * Q / (static_cast<double>(tiles) * TALL_BM);
            if (eff > best + 1e-9 || (eff > best - 1e-9 && tw > btw)) {
                best = eff;
                bth = th;
                btw = tw;
            }
        }
    }
    if (bth == 0) return false;
    *th_out = bth;
    *tw_out = btw;
    *eff_out = best;
    return true;
}

}  // namespace

bool tall_eligible(const ConvParams &p, bool vec, int *th, int *tw, double *eff, bool pool2) {
    if (pool2 && (p.P % 2 != 0 || p.Q % 2 != 0 || p.res || !p.relu || !p.vec_store || p.K % 8 != 0)) return false;
    return vec && p.ldx == p.C && p.R == 3 && p.S == 3 && p.stride == 1 && p.pad == 1 && p.C % BK == 0 && p.P == p.H &&
           p.Q == p.W && tall_geometry(p.P, p.Q, pool2, th, tw, eff);
}

long long tall_tiles(const ConvParams &p, int th, int tw) {
    return 1LL * p.N * ((p.P + th - 1) / th) * ((p.Q + tw - 1) / tw) * ((p.K + TALL_BN - 1) / TALL_BN);
}

hipError_t launch_tall(ConvParams p, int th, int tw, bool pool2, hipStream_t stream) {
    if (pool2 && (th % 2 != 0 || tw % 2 != 0)) return hipErrorInvalidValue;
    p.pool2 = pool2 ? 2 : 0;
    p.th = th;
    p.tw = tw;
    p.n_cb = (p.Q + tw - 1) / tw;                       // tiles per tile row
    p.tiles_img = p.n_cb * ((p.P + th - 1) / th);       // tiles per image
    p.tiles_n = (p.K + TALL_BN - 1) / TALL_BN;
    p.n_tiles = p.N * p.tiles_img * p.tiles_n;
    p.split_k = 1;
    p.tiles_per_xcd = (p.n_tiles + 7) / 8;
    p.d_tiles_n = make_fastdiv(p.tiles_n);
    p.d_tw = make_fastdiv(tw);
    p.d_ncb = make_fastdiv(p.n_cb);
    p.d_pwt = make_fastdiv(tw + 2);
    p.d_hp = make_fastdiv(p.tiles_img);
    if (p.stamps)
        hipLaunchKernelGGL(conv3x3_tall_kernel<true>, dim3(static_cast<unsigned>(p.tiles_per_xcd * 8)), dim3(12 * 64), 0, stream, p);
    else
        hipLaunchKernelGGL(conv3x3_tall_kernel<false>, dim3(static_cast<unsigned>(p.tiles_per_xcd * 8)), dim3(12 * 64), 0, stream, p);
    return hipGetLastError();
}

}  // namespace conv
}  // namespace gpulet
