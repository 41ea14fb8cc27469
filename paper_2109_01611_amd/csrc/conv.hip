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
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>

#include "gpulet_internal.h"

namespace gpulet {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

typedef __attribute__((ext_vector_type(2))) short s16x2;

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
// Two floats -> two bf16 (round to nearest even) in one dword, the first in the low half.
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
    const f32x2 v = {lo, hi};
    const bf16x2 h = __builtin_convertvector(v, bf16x2);
    return *reinterpret_cast<const unsigned *>(&h);
}

constexpr int BK = 64;         // depth slice per main-loop step (elements)
constexpr int CHUNK = 8;       // elements per 16-byte chunk
constexpr int NTHREADS = 256;  // scalar-gather variant: four wavefronts
constexpr unsigned OOB = 0x80000000u;      // byte offset past every buffer: the load returns zeros
constexpr int RSRC_FLAGS = 0x00020000;     // raw buffer descriptor, 32-bit data format

// Division of a non-negative int below 2^30 by a fixed positive divisor through one 64-bit
// multiply: q = (n * mul) >> shift with shift = 30 + ceil(log2 d), mul = floor(2^shift / d) + 1.
// Exact because n * (mul * d - 2^shift) <= n * d < 2^shift.  The tile setup of these kernels is
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

struct ConvParams {
    const __bf16 *x, *w;
    const float *b;
    __bf16 *y;
    const __bf16 *res;
    int N, C, H, W, K, R, S, stride, pad, relu, P, Q;
    int M, Kg;          // GEMM rows and depth
    int ldy, y_off;     // channels per output pixel of the destination, first channel
    int tiles_n, n_tiles, tiles_per_xcd;
    unsigned x_bytes, w_bytes;
    int tap_inner;      // depth order: 64-channel block outermost, filter taps inside it
    int vec_store;      // output (and residual) rows allow aligned 16-byte accesses
    int split_k;        // workgroups sharing one output tile, each taking a contiguous range of slices
    int sps;            // slices per split
    float *part;        // split-K scratch: [n_tiles * split_k][BM * BN] fp32 partial tiles
    unsigned *cnt;      // split-K scratch: arrival counter per tile (zero between launches)
    // Patch kernel only: output pixels are grouped in column blocks of `tw` pixels.
    int tw, n_cb;       // block width, blocks per output row
    FastDiv d_pq, d_q, d_p, d_tiles_n, d_split_k, d_c, d_s;   // by P*Q, Q, P, tiles_n, split_k, C, S
    FastDiv d_tw, d_ncb, d_pwt, d_hp;                         // patch kernel: by tw, n_cb, tw + 2, H + 2*pad
};

// LDS position (in elements) of chunk `chunk` of row `row` in a [rows][BK] tile.
// Rows are 128 bytes; XOR-ing the chunk index with bits 1..3 of the row spreads
// 16 consecutive rows at one logical chunk over all 64 banks.
__device__ __forceinline__ int lds_pos(int row, int chunk) {
    return row * BK + ((chunk ^ ((row >> 1) & 7)) * CHUNK);
}

// Workgroups are dealt round-robin to the eight dies, each with its own L2.
// Give every die a contiguous run of tiles so that tiles sharing a pixel block
// (all their channel tiles) hit the same L2.
__device__ __forceinline__ int tile_of_block(const ConvParams &p) {
    return (blockIdx.x & 7) * p.tiles_per_xcd + (blockIdx.x >> 3);
}

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
typedef __attribute__((ext_vector_type(4))) int i32x4;

// s_waitcnt immediate that waits until at most n vector-memory operations are
// outstanding and leaves the other counters alone (gfx9 encoding).
constexpr int vmcnt_imm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

// Raw buffer descriptor over `bytes` bytes at `ptr`: offsets at or past `bytes` read as zero.
__device__ __forceinline__ i32x4 make_rsrc(const void *ptr, unsigned bytes) {
    const unsigned long long a = reinterpret_cast<unsigned long long>(ptr);
    return i32x4{static_cast<int>(a), static_cast<int>((a >> 32) & 0xFFFF), static_cast<int>(bytes), RSRC_FLAGS};
}

// LDS byte address of a __shared__ object.
__device__ __forceinline__ unsigned lds_addr(const void *p) {
    return static_cast<unsigned>(reinterpret_cast<unsigned long long>(
        (const __attribute__((address_space(3))) char *)p));
}

// One wavefront-wide transfer of 64 x 16 bytes from a buffer into LDS: lane i's
// 16 bytes at byte offset `voff` land at LDS address `lds_base` + 16*i
// (`lds_base` is the same for the whole wavefront and travels in M0).  Issued
// as assembly so that waiting for it stays under this kernel's control: the
// transfers of later ring stages must remain in flight across LDS reads.
__device__ __forceinline__ void dma16(const i32x4 rsrc, unsigned lds_base, unsigned voff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_base), "v"(voff), "s"(rsrc)
                 : "memory");
}

// Last step of the epilogue for a BM x BN fp32 tile parked in LDS (rows padded
// to BN + 8 floats): every thread of the workgroup takes 8 consecutive channels
// of one tile row at a time, adds bias and residual, applies ReLU, rounds once
// to bf16 and stores 16 bytes.  `pixel_of(row)` gives the output pixel
// (n*P + p)*Q + q of a tile row, or -1 for rows past the end.  A thread keeps
// its channel group for all of its rows, so the bias is loaded once, and the
// residual loads of all its rows are issued before the first store: layers with
// a short depth are bound by this loop, and one load-use-store chain per row
// would leave it waiting for memory latency several times per tile.
// The bias of the 8 channels a thread handles in finish_tile.  Called at the very start of a
// kernel, so that the load's latency is hidden behind the whole main loop instead of sitting
// between the last barrier and the first store.
struct BiasRegs {
    float4 lo, hi;
};

template <int BN, int NTHR>
__device__ __forceinline__ BiasRegs load_bias(const ConvParams &p, int n0) {
    constexpr int VPR = BN / 8;
    const int k = n0 + (threadIdx.x % VPR) * 8;
    BiasRegs r;
    r.lo = r.hi = make_float4(0.f, 0.f, 0.f, 0.f);
    if (p.b && p.vec_store && k + 8 <= p.K) {
        r.lo = *reinterpret_cast<const float4 *>(p.b + k);
        r.hi = *reinterpret_cast<const float4 *>(p.b + k + 4);
    }
    return r;
}

template <int BM, int BN, int NTHR, typename PixelOf>
__device__ __forceinline__ void finish_tile(const ConvParams &p, const float *stg, int n0, const BiasRegs &br,
                                            PixelOf pixel_of) {
    constexpr int LDT = BN + 8;
    constexpr int VPR = BN / 8;            // 8-channel groups per tile row
    constexpr int RSTEP = NTHR / VPR;      // tile rows between two items of a thread
    constexpr int ITEMS = (BM + RSTEP - 1) / RSTEP;
    static_assert(NTHR % VPR == 0, "a thread keeps its channel group");
    if (!(p.vec_store && p.K % 8 == 0)) {
        // Destinations that do not allow aligned 16-byte stores (channel counts such as the 546
        // of a detection head, odd channel offsets): one element per thread and pass, with the
        // lanes of a wavefront on consecutive channels of one pixel, so that the 2-byte stores
        // of an instruction fall into one or two 128-byte lines; the bias is loaded once.
        static_assert(NTHR % BN == 0, "whole tile rows per pass");
        constexpr int ROWS = NTHR / BN;
        const int c = threadIdx.x % BN, kc = n0 + c;
        if (kc >= p.K) return;
        const float bias1 = p.b ? p.b[kc] : 0.f;
        for (int row = threadIdx.x / BN; row < BM; row += ROWS) {
            const int m = pixel_of(row);
            if (m < 0) continue;
            float a = stg[row * LDT + c] + bias1;
            if (p.res) a += static_cast<float>(p.res[m * p.K + kc]);
            if (p.relu) a = a > 0.f ? a : 0.f;
            p.y[m * p.ldy + p.y_off + kc] = static_cast<__bf16>(a);
        }
        return;
    }
    const int cv = threadIdx.x % VPR, row0 = threadIdx.x / VPR;
    const int k = n0 + cv * 8;
    if (k >= p.K) return;
    {
        const float bias[8] = {br.lo.x, br.lo.y, br.lo.z, br.lo.w, br.hi.x, br.hi.y, br.hi.z, br.hi.w};
        const unsigned limit = relu_limit(p.relu);
        int m[ITEMS];
        uint4 rr[ITEMS];
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const int row = row0 + i * RSTEP;
            m[i] = row < BM ? pixel_of(row) : -1;
            rr[i] = make_uint4(0u, 0u, 0u, 0u);
        }
        if (p.res) {
#pragma unroll
            for (int i = 0; i < ITEMS; ++i)
                if (m[i] >= 0) rr[i] = *reinterpret_cast<const uint4 *>(p.res + (m[i] * p.K + k));
        }
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            if (m[i] < 0) continue;
            const int row = row0 + i * RSTEP;
            const float4 lo = *reinterpret_cast<const float4 *>(&stg[row * LDT + cv * 8]);
            const float4 hi = *reinterpret_cast<const float4 *>(&stg[row * LDT + cv * 8 + 4]);
            float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] += bias[e];
            if (p.res) {
                // a bf16 is the upper half of the fp32 with the same value
                const unsigned ru[4] = {rr[i].x, rr[i].y, rr[i].z, rr[i].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[2 * e] += __uint_as_float(ru[e] << 16);
                    v[2 * e + 1] += __uint_as_float(ru[e] & 0xFFFF0000u);
                }
            }
            unsigned pk[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                pk[e] = relu_or_pass(pack_bf16(v[2 * e], v[2 * e + 1]), limit);
            *reinterpret_cast<uint4 *>(p.y + (m[i] * p.ldy + p.y_off + k)) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        }
    }
}

// Wavefronts are specialised.  The first CWM x CWN wavefronts ("consumers")
// only read LDS and issue MFMAs; the last NPROD wavefronts ("producers") only
// compute addresses and issue transfers.  A wavefront blocked on a saturated
// memory pipeline therefore never holds back matrix instructions.  Every ring
// step has one workgroup barrier: before it a producer waits for its own
// transfers of slice j, after it the stage slice j-1 occupied is free again.
template <int BM, int BN, int CWM, int CWN, int NPROD, int NS, bool POINTWISE>
__global__ __launch_bounds__((CWM * CWN + NPROD) * 64) void conv_igemm_kernel(const ConvParams p) {
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
    const int item = tile_of_block(p);
    if (item >= p.n_tiles * p.split_k) return;
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
                a_off[i] = (((n * p.H + a_h0[i]) * p.W + a_w0[i]) * p.C) * 2;
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
        // Advancing s by one and c by -C leaves the address unchanged (a filter row
        // covers a contiguous span of the image row), so the offset only jumps when
        // the filter moves to its next row.
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
            tap = ((r * p.W + s) * p.C + c) * 2;
        } else {
            g = k_first * BK + cc * CHUNK;
            const int t = fdiv(g, p.d_c);
            c = g - t * p.C;
            r = fdiv(t, p.d_s);
            s = t - r * p.S;
            tap = ((r * p.W + s) * p.C + c) * 2;
        }
        auto normalise = [&]() {
            while (c >= p.C) {
                c -= p.C;
                if (++s == p.S) {
                    s = 0;
                    ++r;
                    tap += (p.W - p.S) * p.C * 2;
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
                tap += p.C * 2;
                if (++s == p.S) {
                    s = 0;
                    tap += (p.W - p.S) * p.C * 2;
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
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
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
    finish_tile<BM, BN, NTHR>(p, stg, n0, bias_regs, [&](int row) { return m0 + row < p.M ? m0 + row : -1; });
}

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
// lane.  Each position is a 128-byte row of 64 channels, XOR-swizzled like the
// weight tiles (by the position index).  The host guarantees that no tile
// needs more than PMAX positions.
//
// Four consumer wavefronts (one per SIMD) own 32 tile rows x 64 channels each;
// four producers issue the transfers.  Patch buffers alternate per channel
// block, weight stages form a ring of three.  A producer's transfers complete
// in issue order, which the waits below rely on: within a step the pieces of
// the next patch are issued before the weights of step t+2, so waiting for the
// weights of step t also covers every patch piece issued earlier.
// ---------------------------------------------------------------------------
constexpr int PATCH_BM = 128;
constexpr int PATCH_PMAX = 256;  // patch positions per buffer (32 KB)

template <int BN, int NPROD>
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
    __bf16 *const patch = lds;
    __bf16 *const wring = lds + 2 * PATCH;

    const int tile = tile_of_block(p);
    if (tile >= p.n_tiles) return;
    const int tm = fdiv(tile, p.d_tiles_n), tn = tile - tm * p.tiles_n;
    const int tl = fdiv(tm, p.d_ncb), cb = tm - tl * p.n_cb;
    const int l0 = tl * BM, n0 = tn * BN, q0 = cb * p.tw;
    const BiasRegs bias_regs = load_bias<BN, (NCONS + NPROD) * 64>(p, n0);
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

        // Patch transfer j of this wavefront fills positions (j*NPROD + pw)*8 .. +8;
        // this lane fills physical chunk lane&7 of one of them.
        unsigned a_off[POPS];
#pragma unroll
        for (int j = 0; j < POPS; ++j) {
            const int pos = (j * NPROD + pw) * 8 + (lane >> 3);
            const int cc = (lane & 7) ^ ((pos >> 1) & 7);
            a_off[j] = OOB;
            if (pos < npos) {
                const int vr = fdiv(pos, p.d_pwt), u = pos - vr * pwt;
                const int v = v0 + vr;
                const int n = fdiv(v, p.d_hp);
                const int h = v - n * Hp - p.pad, w = q0 + u - p.pad;
                if (n < p.N && (unsigned)h < (unsigned)p.H && (unsigned)w < (unsigned)p.W)
                    a_off[j] = static_cast<unsigned>((((n * p.H + h) * p.W + w) * p.C + cc * CHUNK) * 2);
            }
        }
        // Weight transfer i fills rows rg*8 .. +8 of tap s of the stage, q = i*NPROD + pw = s*RG + rg.
        unsigned b_off[BOPS];
#pragma unroll
        for (int i = 0; i < BOPS; ++i) {
            const int q = i * NPROD + pw;
            const int s = q / RG, row = (q - s * RG) * 8 + (lane >> 3);
            const int cc = (lane & 7) ^ ((row >> 1) & 7);
            const int k = n0 + row;
            b_off[i] = k < p.K ? static_cast<unsigned>(((k * 9 + s) * p.C + cc * CHUNK) * 2) : OOB;
        }

        auto issue_patch = [&](int blk, int half) {
            const unsigned base = lds_addr(patch + (blk & 1) * PATCH) + pw * 1024;
            const unsigned add = static_cast<unsigned>(blk * BK * 2);
#pragma unroll
            for (int j = half * (POPS / 2); j < (half + 1) * (POPS / 2); ++j) {
                const unsigned off = (blk < nblk && a_off[j] != OOB) ? a_off[j] + add : OOB;
                dma16(rx, base + j * NPROD * 1024, off);
            }
        };
        // Weights of step t = 3*blk + r into ring stage `stage`.
        auto issue_weights = [&](int blk, int r, int stage) {
            const unsigned base = lds_addr(wring + stage * BSTAGE) + pw * 1024;
            const unsigned add = static_cast<unsigned>((r * 3 * p.C + blk * BK) * 2);
#pragma unroll
            for (int i = 0; i < BOPS; ++i) {
                const unsigned off = (blk < nblk && b_off[i] != OOB) ? b_off[i] + add : OOB;
                dma16(rw, base + i * NPROD * 1024, off);
            }
        };

        issue_patch(0, 0);
        issue_patch(0, 1);
        issue_weights(0, 0, 0);
        issue_weights(0, 1, 1);
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
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

        // Patch position of this lane's tile row at tap (0, 0).
        int base = 0;
        {
            const int l = l0 + wave * 32 + frow;
            const int rho = fdiv(l, p.d_tw);
            if (rho < NP) base = (vrow(rho) - v0) * pwt + (l - rho * p.tw);
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
                const __bf16 *wb = wring + r * BSTAGE;
                auto load = [&](Frags &f, int i) {
                    const int s = i / (BK / 16), ks = i % (BK / 16);
                    const int pos = base + r * pwt + s;
                    f.a = *reinterpret_cast<const bf16x8 *>(pa + pos * BK +
                                                            (((ks * 2 + fhalf) ^ ((pos >> 1) & 7)) * CHUNK));
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
    finish_tile<BM, BN, (NCONS + NPROD) * 64>(p, stg, n0, bias_regs, [&](int row) {
        const int l = l0 + row;
        const int rho = fdiv(l, p.d_tw);
        const int q = q0 + (l - rho * p.tw);
        return (rho < NP && q < p.Q) ? rho * p.Q + q : -1;
    });
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
__global__ __launch_bounds__(512) void conv3x3_c64_kernel(const ConvParams p, const int wgs_per_col, const int tiles_m,
                                                          const int die_aware) {
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
    const int NP = p.N * p.P;
    const int Hp = p.H + 2 * p.pad;       // virtual rows per image
    const int pwt = p.tw + 2;             // patch width: block columns plus the two halo columns
    if (threadIdx.x < BN) lbias[threadIdx.x] = (p.b && n0 + threadIdx.x < p.K) ? p.b[n0 + threadIdx.x] : 0.f;

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
                const int cc = (lane & 7) ^ ((pos >> 1) & 7);
                unsigned off = OOB;
                if (pos < tl.npos) {
                    const int vr = fdiv(pos, p.d_pwt), u = pos - vr * pwt;
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
        unsigned char *tr = trs + wave * (64 * TROW);
        const unsigned limit = relu_limit(p.relu);
        const int kst = n0 + wx * 32 + (lane & 3) * 8;   // first of the 8 filters this lane stores

        for (int t = 0; t < T; ++t) {
            const Tile tl = tile_at(t);
            // Patch positions of this lane's two pixels at tap (0, 0).
            int base[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int l = tl.l0 + wy * 64 + i * 32 + frow;
                const int rho = fdiv(l, p.d_tw);
                base[i] = rho < NP ? (vrow(rho) - tl.v0) * pwt + (l - rho * p.tw) : 0;
            }
            f32x16 acc[2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
            __syncthreads();  // B1
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
                    f.a[h] = *reinterpret_cast<const bf16x8 *>(pa + pos * BK + (((ks * 2 + fhalf) ^ ((pos >> 1) & 7)) * CHUNK));
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
            __syncthreads();  // B2

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
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }
}

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
                const unsigned off = k < p.K ? static_cast<unsigned>((k * p.C + q * BK + cc * CHUNK) * 2) : OOB;
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
                    dma16(rx, base + (q * BM + i * PROWS) * (BK * 2), pix == OOB ? OOB : pix + q * (BK * 2));
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

__device__ __forceinline__ unsigned bf16_pair_order_key(unsigned v) {
    const s16x2 x = *reinterpret_cast<const s16x2 *>(&v);
    const s16x2 k = x ^ ((x >> 15) & static_cast<short>(0x7fff));
    return *reinterpret_cast<const unsigned *>(&k);
}
__device__ __forceinline__ unsigned max_keys(unsigned a, unsigned b) {
    const s16x2 r = __builtin_elementwise_max(*reinterpret_cast<const s16x2 *>(&a), *reinterpret_cast<const s16x2 *>(&b));
    return *reinterpret_cast<const unsigned *>(&r);
}

// These layers are small (a few hundred pixel tiles at most) and all latency: a tile is 32
// pixels x 64 filters so that there are enough workgroups, every thread pools one chunk per
// slice, and the raw loads of slices j+1 and j+2 are in flight while slice j is multiplied.
// Only two of the four wavefronts issue matrix instructions (32 x 32 each); all four load.
__global__ __launch_bounds__(256) void pooled_conv1x1_kernel(const ConvParams p) {
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
            a_base[i] = ((n * p.H + a_h0[i]) * p.W + a_w0[i]) * p.C;
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
            const int tap = (r * p.W + s) * p.C + c;
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
    const dim3 grid(static_cast<unsigned>(p.tiles_per_xcd * 8));
    const dim3 block((CWM * CWN + NPROD) * 64);
    const bool pointwise = p.R == 1 && p.S == 1 && p.pad == 0;
    if (vec && pointwise)
        hipLaunchKernelGGL((conv_igemm_kernel<BM, BN, CWM, CWN, NPROD, NS, true>), grid, block, 0, stream, p);
    else if (vec)
        hipLaunchKernelGGL((conv_igemm_kernel<BM, BN, CWM, CWN, NPROD, NS, false>), grid, block, 0, stream, p);
    else
        hipLaunchKernelGGL((conv_igemm_any_kernel<BM, BN, WGM, WGN>), grid, dim3(NTHREADS), 0, stream, p);
    return hipGetLastError();
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

bool patch_eligible(const ConvParams &p, bool vec, int *tw_out) {
    return vec && p.R == 3 && p.S == 3 && p.stride == 1 && p.pad == 1 && p.C % BK == 0 && p.P == p.H &&
           p.Q == p.W && patch_geometry(p, tw_out);
}

template <int BN>
hipError_t launch_patch(ConvParams p, int tw, hipStream_t stream) {
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
    hipLaunchKernelGGL((conv3x3_patch_kernel<BN, 4>), dim3(static_cast<unsigned>(p.tiles_per_xcd * 8)),
                       dim3(8 * 64), 0, stream, p);
    return hipGetLastError();
}

// The 3x3 kernel with register-resident weights: what the patch kernel needs, exactly 64 input
// channels, no residual operand, aligned 16-byte stores.
bool c64_applicable(const ConvParams &p, bool vec, int *tw_out) {
    return patch_eligible(p, vec, tw_out) && p.C == BK && !p.res && p.vec_store && p.K % 8 == 0;
}

hipError_t launch_c64(ConvParams p, int tw, int n_cu, hipStream_t stream) {
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
    hipLaunchKernelGGL(conv3x3_c64_kernel, dim3(static_cast<unsigned>(wgs_per_col * p.tiles_n)), dim3(512), 0, stream, p,
                       wgs_per_col, tiles_m, die_aware);
    return hipGetLastError();
}

// The streaming 1x1 kernel: C of 64 or 128, unit filter, enough pixel tiles that every
// workgroup walks over several of them.
bool stream_applicable(const ConvParams &p, bool vec) {
    return vec && p.R == 1 && p.S == 1 && p.pad == 0 && (p.C == 64 || p.C == 128);
}

// Chosen automatically for one depth slice (C = 64: two workgroups per CU) and at least four tiles
// per CU, where it measured 11 % faster than the best one-tile-per-workgroup tile (1x1 64->256 on
// 56x56 at batch 32: 20.3 -> 18.0 us); with two slices (C = 128) it was 8 % slower.
bool stream_eligible(const ConvParams &p, bool vec, int n_cu) {
    const long long tiles = 1LL * ((p.M + STREAM_BM - 1) / STREAM_BM) * ((p.K + STREAM_BN - 1) / STREAM_BN);
    return stream_applicable(p, vec) && p.C == 64 && tiles >= 4LL * n_cu;
}

hipError_t launch_stream(ConvParams p, int n_cu, hipStream_t stream) {
    const int tiles_m = (p.M + STREAM_BM - 1) / STREAM_BM;
    p.tiles_n = (p.K + STREAM_BN - 1) / STREAM_BN;
    p.n_tiles = tiles_m * p.tiles_n;
    p.split_k = 1;
    // two workgroups per CU with one depth slice (75 KB of LDS each), one with two (115 KB)
    const int slots = n_cu * (p.C == 64 ? 2 : 1);
    const int wgs_per_col = std::max(1, std::min(tiles_m, slots / p.tiles_n));
    const dim3 grid(static_cast<unsigned>(wgs_per_col * p.tiles_n));
    if (p.C == 64)
        hipLaunchKernelGGL(conv1x1_stream_kernel<1>, grid, dim3(12 * 64), 0, stream, p, wgs_per_col, tiles_m);
    else
        hipLaunchKernelGGL(conv1x1_stream_kernel<2>, grid, dim3(12 * 64), 0, stream, p, wgs_per_col, tiles_m);
    return hipGetLastError();
}

// The stem kernel: at most four channels, a filter row of at most eight pixels, 3, 5 or 7
// filter rows, a tile's input patch within the staged limit, 16-byte stores possible, no residual.
bool stem_applicable(const ConvParams &p) {
    if (p.C > 4 || p.S > 8 || !(p.R == 3 || p.R == 5 || p.R == 7)) return false;
    if (!p.vec_store || p.K % 8 != 0 || p.res) return false;
    if (p.C == 4 && reinterpret_cast<uintptr_t>(p.x) % 8 != 0) return false;  // 8-byte pixel loads
    const int krow = p.S <= 4 ? 16 : 32;
    const int nrows = (STEM_TP - 1) * p.stride + p.R, ncols = (STEM_TQ - 1) * p.stride + krow / 4;
    return nrows * ncols <= STEM_PX;
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

// Off by default: the partial tiles cross dies through memory, which costs about 8 us per
// launch on MI355X and only pays for layers with very few tiles and a very long depth.
std::atomic<int> g_max_split_k{1};

std::atomic<int> g_tile_override{-1};

struct TileChoice {
    int bm, bn;
    float eff;  // relative MFMA efficiency of the tile shape (bigger tiles reuse LDS reads more)
};

}  // namespace

gpulet_status check_conv(const ConvArgs &a) {
    if (!a.x || !a.w || !a.y) return GPULET_EINVAL;
    if (a.N < 1 || a.C < 1 || a.H < 1 || a.W < 1 || a.K < 1 || a.R < 1 || a.S < 1 || a.stride < 1 ||
        a.pad < 0)
        return GPULET_EINVAL;
    if (a.P < 1 || a.Q < 1) return GPULET_EINVAL;
    if (a.y_ch_offset < 0 || a.y_ch_offset + a.K > a.y_ch_stride) return GPULET_EINVAL;
    if (a.pre_pool != 0 && (a.pre_pool != 3 || a.R != 1 || a.S != 1 || a.stride != 1 || a.pad != 0 || a.C % 8 != 0))
        return GPULET_EINVAL;
    // Byte offsets are 32-bit with the top bit reserved as the out-of-range marker.
    const long long lim = 1LL << 30;
    const long long xe = 1LL * a.N * a.H * a.W * a.C;
    const long long we = 1LL * a.K * a.R * a.S * a.C;
    const long long ye = 1LL * a.N * a.P * a.Q * a.y_ch_stride;
    // The gather indexes from (h, w) = (-pad, -pad) and may step past the last tap.
    const long long slack = (1LL * (a.pad + a.R) * a.W + a.pad + a.S) * a.C + 64;
    if (xe + slack >= lim || we + 64 >= lim || ye >= lim) return GPULET_EINVAL;
    return GPULET_OK;
}

hipError_t launch_conv(const ConvArgs &a, const LaunchCtx &ctx, hipStream_t stream) {
    ConvParams p;
    p.x = static_cast<const __bf16 *>(a.x);
    p.w = static_cast<const __bf16 *>(a.w);
    p.b = a.b;
    p.y = static_cast<__bf16 *>(a.y);
    p.res = static_cast<const __bf16 *>(a.residual);
    p.N = a.N; p.C = a.C; p.H = a.H; p.W = a.W; p.K = a.K; p.R = a.R; p.S = a.S;
    p.stride = a.stride; p.pad = a.pad; p.relu = a.relu; p.P = a.P; p.Q = a.Q;
    p.M = a.N * a.P * a.Q;
    p.Kg = a.R * a.S * a.C;
    p.ldy = a.y_ch_stride;
    p.y_off = a.y_ch_offset;
    p.tiles_n = p.n_tiles = p.tiles_per_xcd = 0;
    p.x_bytes = static_cast<unsigned>(2LL * a.N * a.H * a.W * a.C);
    p.w_bytes = static_cast<unsigned>(2LL * a.K * a.R * a.S * a.C);
    p.tap_inner = (a.C % BK == 0 && a.R * a.S > 1) ? 1 : 0;
    p.vec_store = (a.y_ch_stride % 8 == 0 && a.y_ch_offset % 8 == 0 && reinterpret_cast<uintptr_t>(a.y) % 16 == 0 &&
                   reinterpret_cast<uintptr_t>(a.b) % 16 == 0 &&
                   (!a.residual || (a.K % 8 == 0 && reinterpret_cast<uintptr_t>(a.residual) % 16 == 0)))
                      ? 1
                      : 0;
    p.split_k = 1;
    p.sps = 0;
    p.part = ctx.scratch;
    p.cnt = ctx.counters;
    p.tw = p.n_cb = 0;
    p.d_pq = make_fastdiv(a.P * a.Q);
    p.d_q = make_fastdiv(a.Q);
    p.d_p = make_fastdiv(a.P);
    p.d_c = make_fastdiv(a.C);
    p.d_s = make_fastdiv(a.S);
    p.d_tiles_n = p.d_split_k = p.d_tw = p.d_ncb = p.d_pwt = p.d_hp = make_fastdiv(1);

    const bool vec = (a.C % CHUNK == 0) && (reinterpret_cast<uintptr_t>(a.x) % 16 == 0) &&
                     (reinterpret_cast<uintptr_t>(a.w) % 16 == 0);
    if (a.pre_pool) {
        // checked by check_conv: 3x3 window, 1x1 filter, stride 1, no padding, C % 8 == 0; the
        // callers check the 16-byte alignment of x and w
        if (!vec) return hipErrorInvalidValue;
        return launch_pooled_conv(p, stream);
    }

    // Pick the tile and the split of the depth that minimise
    //   (work items on the busiest CU) x (tile area) x (share of the depth + fixed cost of a split) / efficiency.
    // The efficiencies are measured throughput ratios on MI355X (large layers, all CUs busy);
    // on a tie the earlier entry wins.  A split needs the gpu-let's scratch, at least four
    // slices per workgroup, and pays for parking and re-reading fp32 partial tiles.
    static const TileChoice kTiles[] = {{128, 128, 0.90f}, {128, 64, 0.72f}, {64, 128, 0.72f}, {64, 64, 0.58f},
                                        {128, 32, 0.30f},  {32, 128, 0.40f}, {256, 128, 1.00f}};
    static const int kOrder[] = {6, 0, 2, 1, 3, 5, 4};
    const int nk = (p.Kg + BK - 1) / BK;
    const int forced = g_tile_override.load();
    const int max_split = (vec && ctx.scratch && forced < 0) ? g_max_split_k.load() : 1;
    int best = 0, best_split = 1;
    double best_cost = 0.0;
    const int n_cu = ctx.n_cu < 1 ? 1 : ctx.n_cu;
    for (int o = 0; o < static_cast<int>(sizeof(kOrder) / sizeof(kOrder[0])); ++o) {
        const int i = kOrder[o];
        const TileChoice &t = kTiles[i];
        const long long tiles = 1LL * ((p.M + t.bm - 1) / t.bm) * ((p.K + t.bn - 1) / t.bn);
        for (int sk = 1; sk <= max_split; ++sk) {
            if (sk > 1) {
                const int sps = (nk + sk - 1) / sk;
                if (sps < 4 || (sk - 1) * sps >= nk) continue;                         // too thin, or an empty split
                if (tiles > ctx.n_counters) continue;
                if (static_cast<size_t>(tiles) * sk * t.bm * t.bn * 4 > ctx.scratch_bytes) continue;
            }
            const long long per_cu = (tiles * sk + n_cu - 1) / n_cu;
            const double share = 1.0 / sk + (sk > 1 ? 0.06 + 0.02 * sk : 0.0);
            double eff = t.eff;
            // 128x128 runs two workgroups per CU when there are more tiles than CUs (see the
            // launch below); the overlap of one's loads with the other's epilogue weighs more
            // the shorter the depth (measured against 256x128 at 9 .. 72 slices).
            if (i == 0 && sk == 1 && tiles > n_cu) eff = std::min(1.2, 0.90 + 3.0 / nk);
            const double cost = static_cast<double>(per_cu) * t.bm * t.bn * share / eff;
            if ((o == 0 && sk == 1) || cost < best_cost) {
                best = i;
                best_split = sk;
                best_cost = cost;
            }
        }
    }
    if (forced >= 0 && forced < GPULET_CONV_TILES) {
        best = forced;
        best_split = 1;
    }
    int tw = 0;
    const bool patch_ok = patch_eligible(p, vec, &tw);
    if (best == 7 && !patch_ok) best = 1;  // the patch kernel does not apply: same tile shape, gathered
    // The patch kernel runs one workgroup per CU.  Measured on MI355X it beats the gathering
    // tiles when all of its workgroups are resident at once (a second round doubles its time)
    // and the depth is long enough (four or more channel blocks) to amortise loading the
    // first patch.
    if (forced < 0 && patch_ok && p.C >= 4 * BK) {
        const int n_cb = (p.Q + tw - 1) / tw;
        const long long lin = 1LL * p.N * p.P * tw;
        const long long tiles = ((lin + PATCH_BM - 1) / PATCH_BM) * n_cb * ((p.K + 63) / 64);
        // Workgroups are dealt round-robin to 8 dies and, inside a die, to 4 shader engines; a
        // CU holds one workgroup, so every shader engine must have a CU for each of its share.
        const long long per_se = ((tiles + 7) / 8 + 3) / 4;
        if (per_se <= n_cu / 32) {
            best = 7;
            best_split = 1;
        }
    }
    if (best == 8 && !stream_applicable(p, vec)) best = 2;  // same tile shape, one tile per workgroup
    if (forced < 0 && stream_eligible(p, vec, n_cu)) best = 8;
    int tw64 = 0;
    const bool c64_ok = c64_applicable(p, vec, &tw64);
    if (best == 10 && !c64_ok) best = 1;
    // Loading 144 registers of weights per consumer pays from about eight pixel tiles per
    // workgroup on (measured: 3x3 64->64 on 224x224 at batch 32 209 -> 150-160 us, 64->192 on
    // 56x56 36.6 -> 31.7 us; with three tiles per workgroup, 64->64 on 56x56, it is 9 % slower).
    if (forced < 0 && c64_ok) {
        const int n_cb = (p.Q + tw64 - 1) / tw64;
        const long long tiles_m = ((1LL * p.N * p.P * tw64 + PATCH_BM - 1) / PATCH_BM) * n_cb;
        const int tiles_n = (p.K + 63) / 64;
        const int wgs_per_col = std::max(1, n_cu / tiles_n);
        if (tiles_m >= 8LL * wgs_per_col) best = 10;
    }
    if (best == 9 && !stem_applicable(p)) best = 1;
    if (forced < 0 && stem_applicable(p)) best = 9;  // by shape alone: the same bits in every batch and gpu-let
    switch (best) {
        case 10: return launch_c64(p, tw64, n_cu, stream);
        case 9: return launch_stem(p, n_cu, stream);
        case 8: return launch_stream(p, n_cu, stream);
        case 7: return launch_patch<64>(p, tw, stream);
        case 0: {
            // With more tiles than CUs, a two-stage ring (64 KB, two workgroups per CU, one's loads
            // overlapping the other's epilogue) beats the deeper prefetch of three stages.
            const long long tiles = 1LL * ((p.M + 127) / 128) * ((p.K + 127) / 128);
            if (tiles > n_cu && best_split == 1) return launch_tile<128, 128, 4, 2, 4, 2, 2, 2>(p, vec, 1, stream);
            return launch_tile<128, 128, 4, 2, 4, 3, 2, 2>(p, vec, best_split, stream);
        }
        case 1: return launch_tile<128, 64, 4, 2, 4, 3, 2, 2>(p, vec, best_split, stream);
        case 2: return launch_tile<64, 128, 2, 4, 4, 3, 2, 2>(p, vec, best_split, stream);
        case 3: return launch_tile<64, 64, 2, 2, 2, 3, 2, 2>(p, vec, best_split, stream);
        case 4: return launch_tile<128, 32, 4, 1, 2, 3, 4, 1>(p, vec, best_split, stream);
        case 5: return launch_tile<32, 128, 1, 4, 2, 3, 1, 4>(p, vec, best_split, stream);
        default: return launch_tile<256, 128, 4, 2, 4, 3, 2, 2>(p, vec, best_split, stream);
    }
}

void set_conv_split_k(int max_split) { g_max_split_k.store(max_split); }

void set_conv_tile(int tile) { g_tile_override.store(tile); }

}  // namespace gpulet
