// Shared by the convolution kernels of this library (conv_*.hip): layer
// parameters as the kernels see them, the multiply-shift division, the LDS
// swizzle, the DMA-to-LDS transfer, and the common epilogue that turns an fp32
// tile parked in LDS into bf16 rows (bias, residual, ReLU, one rounding).
// Device code; include from .hip files only.
#ifndef GPULET_CONV_COMMON_H
#define GPULET_CONV_COMMON_H

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstddef>

#include "device_util.h"
#include "gpulet_internal.h"
#include "pool_device.h"

namespace gpulet {
namespace conv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
constexpr int BK = 64;         // depth slice per main-loop step (elements)
constexpr int CHUNK = 8;       // elements per 16-byte chunk
constexpr int NTHREADS = 256;  // scalar-gather variant: four wavefronts
constexpr unsigned OOB = 0x80000000u;      // byte offset past every buffer: the load returns zeros
constexpr int RSRC_FLAGS = 0x00020000;     // raw buffer descriptor, 32-bit data format

// The argument block of every convolution kernel.  A kernel fetches only the 64-byte lines of
// it that hold fields it reads, and each line costs a fraction of a microsecond at the start
// of every workgroup, so the fields are ordered by who reads them: lines 0-2 serve every
// kernel, line 3 adds what filters larger than 1x1 and the patch kernels need, the rest is
// for layers with a depth split, a second output or a pooling side job.
struct alignas(64) ConvParams {
    // ---- line 0
    const __bf16 *x, *w;
    const float *b;
    __bf16 *y;
    const __bf16 *res;
    int N, C, H, W, K, R;
    // ---- line 1
    int S, stride, pad, relu, P, Q;
    int M, Kg;          // GEMM rows and depth
    int ldy, y_off;     // channels per output pixel of the destination, first channel
    int ldx;            // channels per input pixel as stored (x points at the layer's first channel);
                        // only the gathering kernels accept ldx != C
    int k2;             // first filter that goes to the second destination (K: there is none)
    int side_blocks;    // workgroups at the end of the grid that run the pooling side job
    int tiles_n, n_tiles, tiles_per_xcd;
    // ---- line 2
    unsigned x_bytes, w_bytes;
    int tap_inner;      // depth order: 64-channel block outermost, filter taps inside it
    int vec_store;      // output (and residual) rows allow aligned 16-byte accesses
    int split_k;        // workgroups sharing one output tile, each taking a contiguous range of slices
    int sps;            // slices per split
    FastDiv d_pq, d_q, d_tiles_n, d_split_k, d_c;   // by P*Q, Q, tiles_n, split_k, C
    // ---- line 3
    FastDiv d_s, d_p;   // by S, P
    // Patch kernels only: output pixels are grouped in column blocks of `tw` pixels.
    int tw, n_cb;       // block width, blocks per output row
    FastDiv d_tw, d_ncb, d_pwt, d_hp;               // by tw, n_cb, tw + 2, H + 2*pad (tall tiles: tiles_img)
    // Tall-tile kernel only: a tile is a th x tw pixel rectangle of one image (n_cb = tiles per
    // tile row, tiles_img = tiles per image).
    int th, tiles_img;
    // ---- line 4 and on
    float *part;        // split-K scratch: [n_tiles * split_k][BM * BN] fp32 partial tiles
    unsigned *cnt;      // split-K scratch: arrival counter per tile (zero between launches)
    // Second destination (1x1 gathering kernels only): filters k >= k2 are stored to
    // y2[m * ldy2 + y2_off + k - k2] instead.
    __bf16 *y2;
    int ldy2, y2_off;
    // Tall-tile kernel only: 2 = a 2x2 / stride 2 max pool follows the layer and only the pooled
    // tensor (N, P/2, Q/2 pixels of ldy channels) is stored to y; 0 = the layer's own output.
    int pool2, pad4;
    // Patch and tall-tile kernels only: when not null, the first kStampWgs workgroups record the
    // wall clock (10 ns units) at kStampPoints points of their life here (gpulet_conv2d_timeline).
    long long *stamps;
    // Side job (1x1 gathering kernels only): the side_blocks extra workgroups compute the
    // 3x3 / stride 1 / pad 1 max pool side_pool of the layer's (dense) input.
    PoolParams side_pool;
};
static_assert(offsetof(ConvParams, S) == 64 && offsetof(ConvParams, x_bytes) == 128 &&
                  offsetof(ConvParams, d_s) == 192 && offsetof(ConvParams, part) == 256,
              "ConvParams: fields grouped by 64-byte line");


// Brings the first four lines of the argument block into registers at once.  Left to itself the
// compiler loads a field where it is first needed, which for a kernel that decodes its tile,
// leaves early when it has none, and then sets up addresses makes three or four dependent round
// trips to memory (the argument block is not cached from one launch to the next), each a few
// hundred nanoseconds in front of the first transfer.  Call first thing in a kernel.
__device__ __forceinline__ void fetch_params(const ConvParams &p) {
    asm volatile("" ::"s"(p.x), "s"(p.w), "s"(p.b), "s"(p.y), "s"(p.res), "s"(p.N), "s"(p.C), "s"(p.H), "s"(p.W), "s"(p.K),
                 "s"(p.R), "s"(p.S), "s"(p.stride), "s"(p.pad), "s"(p.relu), "s"(p.P), "s"(p.Q), "s"(p.M), "s"(p.Kg),
                 "s"(p.ldy), "s"(p.y_off), "s"(p.ldx), "s"(p.k2), "s"(p.tiles_n), "s"(p.n_tiles), "s"(p.tiles_per_xcd),
                 "s"(p.x_bytes), "s"(p.w_bytes), "s"(p.vec_store));
    asm volatile("" ::"s"(p.d_pq.mul), "s"(p.d_pq.shift), "s"(p.d_q.mul), "s"(p.d_q.shift), "s"(p.d_tiles_n.mul),
                 "s"(p.d_tiles_n.shift), "s"(p.d_c.mul), "s"(p.d_c.shift), "s"(p.d_s.mul), "s"(p.d_s.shift),
                 "s"(p.d_p.mul), "s"(p.d_p.shift), "s"(p.tw), "s"(p.n_cb), "s"(p.d_tw.mul), "s"(p.d_tw.shift),
                 "s"(p.d_ncb.mul), "s"(p.d_ncb.shift), "s"(p.d_pwt.mul), "s"(p.d_pwt.shift), "s"(p.d_hp.mul),
                 "s"(p.d_hp.shift), "s"(p.th), "s"(p.tiles_img), "s"(p.tap_inner), "s"(p.split_k), "s"(p.sps));
}

// Wall-clock stamps of a workgroup for the timeline entry point: taken by the first wavefront of
// the first kStampWgs workgroups and stored at once by its first lane.  Only the kernel instances
// compiled with ON record anything (a branch per point cost the ordinary launches 1-4 %); in the
// others every member is empty.
constexpr int kStampWgs = 8, kStampPoints = 8;
template <bool ON>
struct Stamps {
    long long *slot = nullptr;   // this workgroup's row, or null
    __device__ __forceinline__ Stamps(const ConvParams &p, int wave) {
        if constexpr (ON) {
            if (p.stamps != nullptr && blockIdx.x < kStampWgs && wave == 0) slot = p.stamps + blockIdx.x * kStampPoints;
        }
    }
    __device__ __forceinline__ void at(int i) {
        if constexpr (ON) {
            if (slot) {
                const long long t = wall_clock64();
                if (threadIdx.x == 0) slot[i] = t;
            }
        }
    }
    // a stamp taken before this object could be made (before the argument block was there)
    __device__ __forceinline__ void put(int i, long long t) {
        if constexpr (ON) {
            if (slot && threadIdx.x == 0) slot[i] = t;
        }
    }
};

// LDS position (in elements) of chunk `chunk` of row `row` in a [rows][BK] tile.
// Rows are 128 bytes; XOR-ing the chunk index with bits 1..3 of the row spreads
// 16 consecutive rows at one logical chunk over all 64 banks.
__device__ __forceinline__ int lds_pos(int row, int chunk) {
    return row * BK + ((chunk ^ ((row >> 1) & 7)) * CHUNK);
}

// Swizzle key of position `pos` (a 128-byte row of 64 channels) of an input patch whose rows
// are the block columns plus two halo columns, `prow` = pos / (row width): the key follows
// q = pos - 2*prow, which steps by one from an output pixel to the next also where pos skips
// the halo columns between two patch rows.  The skip is odd, so even and odd positions keep
// alternating and each parity sees eight consecutive values of q >> 1: 16 consecutive pixels
// at a tap touch 16 different 16-byte bank groups.
__device__ __forceinline__ int patch_key(int pos, int prow) { return ((pos - 2 * prow) >> 1) & 7; }

// Workgroups are dealt round-robin to the eight dies, each with its own L2.
// Give every die a contiguous run of tiles so that tiles sharing a pixel block
// (all their channel tiles) hit the same L2.
__device__ __forceinline__ int tile_of_block(const ConvParams &p, int bid) {
    return (bid & 7) * p.tiles_per_xcd + (bid >> 3);
}
__device__ __forceinline__ int tile_of_block(const ConvParams &p) { return tile_of_block(p, blockIdx.x); }

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
// M0 is written here without being declared clobbered: the compiler reserves M0 (naming it in a
// clobber list is diagnosed as undefined behaviour) and sets it itself immediately in front of
// every instruction of its own that reads it, none of which these kernels contain (gfx9 LDS
// instructions do not use M0).
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

template <int BM, int BN, int NTHR, bool DUAL = false, typename PixelOf>
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
        __bf16 *yb = p.y + p.y_off + kc;
        int ld = p.ldy;
        if (DUAL && kc >= p.k2) {
            yb = p.y2 + p.y2_off + (kc - p.k2);
            ld = p.ldy2;
        }
        for (int row = threadIdx.x / BN; row < BM; row += ROWS) {
            const int m = pixel_of(row);
            if (m < 0) continue;
            float a = stg[row * LDT + c] + bias1;
            if (p.res) a += static_cast<float>(p.res[m * p.K + kc]);
            if (p.relu) a = a > 0.f ? a : 0.f;
            yb[m * ld] = static_cast<__bf16>(a);
        }
        return;
    }
    const int cv = threadIdx.x % VPR, row0 = threadIdx.x / VPR;
    const int k = n0 + cv * 8;
    if (k >= p.K) return;
    {
        // a thread keeps its 8 channels, so it also keeps its destination
        __bf16 *yb = p.y + p.y_off + k;
        int ld = p.ldy;
        if (DUAL && k >= p.k2) {
            yb = p.y2 + p.y2_off + (k - p.k2);
            ld = p.ldy2;
        }
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
            *reinterpret_cast<uint4 *>(yb + m[i] * ld) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        }
    }
}

// Several independent layers in one launch of the gathering kernel: workgroups first[j] ..
// first[j+1]-1 work on layer j (unused entries of `first` hold INT_MAX).
constexpr int MAX_GROUP = kMaxGroup;
struct ConvGroup {
    ConvParams p[MAX_GROUP];
    int first[MAX_GROUP + 1];
};

// Patch-based 3x3 kernels: pixels per tile and patch positions per LDS buffer (32 KB).
constexpr int PATCH_BM = 128;
constexpr int PATCH_PMAX = 256;

// ---------------------------------------------------------------------------
// Host side of each kernel family: whether it applies to a layer, and its launch.
// `vec` = C % 8 == 0 with 16-byte aligned x and w.
// ---------------------------------------------------------------------------

// conv_igemm.hip: gathering tiles 0..6 of gpulet_set_conv_tile (scalar-gather variant when !vec).
// `two_stage` selects the 64 KB ring of tile 0 (two workgroups per CU).
hipError_t launch_igemm(const ConvParams &p, bool vec, int tile, int split_k, bool two_stage, hipStream_t stream);
// n (2..MAX_GROUP) layers, all with 16-byte gathers, one tile shape, no depth split, one launch.
hipError_t launch_igemm_group(const ConvParams *p, int n, int tile, bool two_stage, hipStream_t stream);

// conv_patch.hip: tile 7 (input patch in LDS) and tile 10 (64 input channels, weights in registers).
bool patch_eligible(const ConvParams &p, bool vec, int *tw_out);
hipError_t launch_patch(ConvParams p, int tw, hipStream_t stream);
bool c64_applicable(const ConvParams &p, bool vec, int *tw_out, bool pool2 = false);
hipError_t launch_c64(ConvParams p, int tw, int n_cu, bool pool2, hipStream_t stream);

// conv_tall.hip: tile 11 (3x3, 224 x 128 tile, input patch in LDS, one tap per ring step).
// `eff` receives the share of tile rows that are pixels for the chosen rectangle th x tw.
bool tall_eligible(const ConvParams &p, bool vec, int *th, int *tw, double *eff, bool pool2 = false);
long long tall_tiles(const ConvParams &p, int th, int tw);
hipError_t launch_tall(ConvParams p, int th, int tw, bool pool2, hipStream_t stream);

// conv_stream.hip: tile 8 (streaming 1x1).
bool stream_applicable(const ConvParams &p, bool vec);
bool stream_eligible(const ConvParams &p, bool vec, int n_cu);
hipError_t launch_stream(ConvParams p, int n_cu, hipStream_t stream);

// conv_stem.hip: tile 9 (at most four input channels).
bool stem_applicable(const ConvParams &p);
hipError_t launch_stem(ConvParams p, int n_cu, hipStream_t stream);

// conv_pooled.hip: 3x3 / stride 1 / pad 1 max pool fused into a 1x1 convolution.
hipError_t launch_pooled_conv(ConvParams p, hipStream_t stream);

}  // namespace conv
}  // namespace gpulet
#endif  // GPULET_CONV_COMMON_H
