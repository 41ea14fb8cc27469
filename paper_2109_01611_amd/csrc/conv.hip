// Convolution layer of the forward pass served on a gpu-let (paper Sec. 5; the
// models of Table 4): argument checks and the choice of kernel.  The kernels
// themselves live in conv_igemm.hip (implicit GEMM with gathered operands, the
// general case), conv_patch.hip (3x3 with the input patch in LDS), conv_stream.hip
// (1x1 with a short depth), conv_stem.hip (at most four input channels) and
// conv_pooled.hip (max pool fused into a 1x1 convolution); conv_common.h holds
// what they share.
#include <atomic>

#include "conv_common.h"

namespace gpulet {

using namespace conv;

namespace {

// Off by default: the partial tiles cross dies through memory, which costs about 8 us per
// launch on MI355X and only pays for layers with very few tiles and a very long depth.
std::atomic<int> g_max_split_k{1};
std::atomic<int> g_pool_fusion{1};

std::atomic<int> g_tile_override{-1};

struct TileChoice {
    int id, bm, bn;
    float eff;  // relative MFMA efficiency of the tile shape (bigger tiles reuse LDS reads more)
};

// The gathering tiles in the order in which they are tried (on a tie the earlier one wins).
// 192x128 and 96x128 exist for the layers whose 128-pixel tiles just miss a whole number of
// rounds on a gpu-let (98 tiles on 96 CUs, 196 on 192): three row tiles per wavefront instead
// of two or four change the tile count enough to save a round.
const TileChoice kTiles[] = {{6, 256, 128, 1.00f}, {12, 192, 128, 0.93f}, {0, 128, 128, 0.90f}, {13, 96, 128, 0.80f},
                             {2, 64, 128, 0.72f},  {1, 128, 64, 0.72f},   {3, 64, 64, 0.58f},   {5, 32, 128, 0.40f},
                             {4, 128, 32, 0.30f}};
constexpr int kNumTiles = static_cast<int>(sizeof(kTiles) / sizeof(kTiles[0]));

bool is_gathering_tile(int id) { return (id >= 0 && id <= 6) || id == 12 || id == 13; }


}  // namespace

gpulet_status check_conv(const ConvArgs &a) {
    if (!a.x || !a.w || !a.y) return GPULET_EINVAL;
    if (a.N < 1 || a.C < 1 || a.H < 1 || a.W < 1 || a.K < 1 || a.R < 1 || a.S < 1 || a.stride < 1 ||
        a.pad < 0)
        return GPULET_EINVAL;
    if (a.P < 1 || a.Q < 1) return GPULET_EINVAL;
    if (a.y2) {
        if (a.k2 < 1 || a.k2 >= a.K || a.R != 1 || a.S != 1 || a.pad != 0 || a.residual || a.pre_pool)
            return GPULET_EINVAL;
        if (a.y2_ch_offset < 0 || a.y2_ch_offset + (a.K - a.k2) > a.y2_ch_stride) return GPULET_EINVAL;
        if (1LL * a.N * a.P * a.Q * a.y2_ch_stride >= (1LL << 30)) return GPULET_EINVAL;
    }
    if (a.y_ch_offset < 0 || a.y_ch_offset + (a.y2 ? a.k2 : a.K) > a.y_ch_stride) return GPULET_EINVAL;
    if (a.pool_y && (a.R != 1 || a.S != 1 || a.pad != 0 || a.pre_pool || a.C % 8 != 0 ||
                     (a.x_ch_stride != 0 && a.x_ch_stride != a.C)))
        return GPULET_EINVAL;
    if (a.post_pool2 != 0 && (a.post_pool2 != 2 || a.P % 2 != 0 || a.Q % 2 != 0 || a.residual || a.y2 || a.pool_y || a.pre_pool))
        return GPULET_EINVAL;
    if (a.pre_pool != 0 && (a.pre_pool != 3 || a.R != 1 || a.S != 1 || a.stride != 1 || a.pad != 0 || a.C % 8 != 0))
        return GPULET_EINVAL;
    const int ldx = a.x_ch_stride ? a.x_ch_stride : a.C;
    if (a.x_ch_offset < 0 || a.x_ch_offset + a.C > ldx) return GPULET_EINVAL;
    if (ldx != a.C && a.pre_pool) return GPULET_EINVAL;
    // Byte offsets are 32-bit with the top bit reserved as the out-of-range marker.
    const long long lim = 1LL << 30;
    const long long xe = 1LL * a.N * a.H * a.W * ldx;
    const long long we = 1LL * a.K * a.R * a.S * a.C;
    const long long ye = 1LL * a.N * a.P * a.Q * a.y_ch_stride;
    // The gather indexes from (h, w) = (-pad, -pad) and may step past the last tap.
    const long long slack = (1LL * (a.pad + a.R) * a.W + a.pad + a.S) * ldx + 64;
    if (xe + slack >= lim || we + 64 >= lim || ye >= lim) return GPULET_EINVAL;
    return GPULET_OK;
}

namespace {

// The kernel's parameter block for one layer (tile-dependent fields are filled in by the
// launchers) and whether its operands allow 16-byte gathers.
hipError_t make_params(const ConvArgs &a, const LaunchCtx &ctx, ConvParams &p, bool &vec) {
    p.ldx = a.x_ch_stride ? a.x_ch_stride : a.C;
    p.x = static_cast<const __bf16 *>(a.x) + a.x_ch_offset;
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
    p.y2 = static_cast<__bf16 *>(a.y2);
    p.k2 = a.y2 ? a.k2 : a.K;
    p.ldy2 = a.y2_ch_stride;
    p.y2_off = a.y2_ch_offset;
    p.pool2 = p.pad4 = 0;
    p.stamps = static_cast<long long *>(a.stamps);
    p.tiles_n = p.n_tiles = p.tiles_per_xcd = 0;
    // up to the last channel the layer reads of the last pixel
    p.x_bytes = static_cast<unsigned>(2LL * ((1LL * a.N * a.H * a.W - 1) * p.ldx + a.C));
    p.w_bytes = static_cast<unsigned>(2LL * a.K * a.R * a.S * a.C);
    p.tap_inner = (a.C % BK == 0 && a.R * a.S > 1) ? 1 : 0;
    p.vec_store = (a.y_ch_stride % 8 == 0 && a.y_ch_offset % 8 == 0 && reinterpret_cast<uintptr_t>(a.y) % 16 == 0 &&
                   reinterpret_cast<uintptr_t>(a.b) % 16 == 0 &&
                   (!a.residual || (a.K % 8 == 0 && reinterpret_cast<uintptr_t>(a.residual) % 16 == 0)) &&
                   (!a.y2 || (a.k2 % 8 == 0 && a.y2_ch_stride % 8 == 0 && a.y2_ch_offset % 8 == 0 &&
                              reinterpret_cast<uintptr_t>(a.y2) % 16 == 0)))
                      ? 1
                      : 0;
    p.split_k = 1;
    p.sps = 0;
    p.part = ctx.scratch;
    p.cnt = ctx.counters;
    p.tw = p.n_cb = p.th = p.tiles_img = 0;
    p.d_pq = make_fastdiv(a.P * a.Q);
    p.d_q = make_fastdiv(a.Q);
    p.d_p = make_fastdiv(a.P);
    p.d_c = make_fastdiv(a.C);
    p.d_s = make_fastdiv(a.S);
    p.d_tiles_n = p.d_split_k = p.d_tw = p.d_ncb = p.d_pwt = p.d_hp = make_fastdiv(1);

    vec = (a.C % CHUNK == 0) && (p.ldx % CHUNK == 0) && (reinterpret_cast<uintptr_t>(p.x) % 16 == 0) &&
                     (reinterpret_cast<uintptr_t>(a.w) % 16 == 0);
    if (a.y2 && !vec) return hipErrorInvalidValue;  // only the 16-byte gathering kernels store to two tensors
    p.side_blocks = 0;
    p.side_pool = PoolParams{};
    if (a.pool_y) {
        if (!vec || reinterpret_cast<uintptr_t>(a.pool_y) % 16 != 0) return hipErrorInvalidValue;
        PoolParams &sp = p.side_pool;
        sp.x = static_cast<const __bf16 *>(a.x);
        sp.y = static_cast<__bf16 *>(a.pool_y);
        sp.N = a.N; sp.C = a.C; sp.H = a.H; sp.W = a.W; sp.P = a.H; sp.Q = a.W; sp.k = 3; sp.stride = 1; sp.pad = 1;
        sp.total = a.N * a.H * a.W * (a.C / 8);
        sp.d_cv = make_fastdiv(a.C / 8);
        sp.d_q = make_fastdiv(a.W);
        sp.d_p = make_fastdiv(a.H);
    }
    return hipSuccess;
}

// Which kernel runs a layer: 0..6 a gathering tile (with `split` workgroups per tile), 7 the
// patch kernel (column block `tw`), 8 the streaming 1x1 kernel, 9 the stem kernel, 10 the
// resident-weight kernel (column block `tw64`).
struct Choice {
    int best, split, tw, tw64, th11, tw11;
    double cost;   // of `best` in the cost model's units when it is a gathering tile or the tall tile, else 0
};

// Cost of a layer on the tall tile in the units of choose_kernel: rounds on the busiest CU x tile
// area / efficiency relative to the 256x128 gathering tile.  The efficiency is fitted to
// measurements on MI355X (3x3 layers of 128..512 channels on 14..112 pixel maps at batch 16 and
// 32, on 64, 128 and 256 CUs): 0.95 when every tile row is a pixel and the depth is long, less a
// share of the rows that are not pixels (they are already in the tile count; what remains is that
// the epilogue and the patch do not shrink with them) and the first loads and the epilogue that
// a short depth does not amortise.
double tall_cost(const ConvParams &p, int th, int tw, double geo, int n_cu) {
    const double eff = 0.95 - 0.35 * (1.0 - geo) - 0.04 / (p.C / BK);
    return static_cast<double>((tall_tiles(p, th, tw) + n_cu - 1) / n_cu) * 224 * 128 / eff;
}

Choice choose_kernel(const ConvParams &p, bool vec, const LaunchCtx &ctx) {
    // Pick the tile and the split of the depth that minimise
    //   (work items on the busiest CU) x (tile area) x (share of the depth + fixed cost of a split) / efficiency.
    // The efficiencies are measured throughput ratios on MI355X (large layers, all CUs busy);
    // on a tie the earlier entry wins.  A split needs the gpu-let's scratch, at least four
    // slices per workgroup, and pays for parking and re-reading fp32 partial tiles.
    const int nk = (p.Kg + BK - 1) / BK;
    const int forced = g_tile_override.load();
    const int max_split = (vec && ctx.scratch && forced < 0) ? g_max_split_k.load() : 1;
    int best = 0, best_split = 1;
    double best_cost = 0.0;
    const int n_cu = ctx.n_cu < 1 ? 1 : ctx.n_cu;
    for (int o = 0; o < kNumTiles; ++o) {
        const TileChoice &t = kTiles[o];
        const int i = t.id;
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
            // (filters larger than 1x1 gain less: 0.92-0.95 measured at 18 and 36 slices)
            if (i == 0 && sk == 1 && tiles > n_cu) eff = std::min(1.2, 0.90 + (p.R * p.S == 1 ? 3.0 : 0.6) / nk);
            const double cost = static_cast<double>(per_cu) * t.bm * t.bn * share / eff;
            if ((o == 0 && sk == 1) || cost < best_cost) {
                best = i;
                best_split = sk;
                best_cost = cost;
            }
        }
    }
    // Filters larger than 1x1 on very few tiles: the two producers of the 64x64 tile, which locate every
    // tap of their pixels themselves, are what such a launch waits for; 64x128 has four and half as
    // many rows per producer.  Measured on MI355X with at most an eighth as many 64x64 tiles as CUs
    // (3x3 stride 2 at batch 1, SSD's last feature maps): 64x128 is 7-10 % faster; from 56 tiles on
    // 256 CUs on it is the other way round or even.
    if (forced < 0 && best == 3 && best_split == 1 && p.R * p.S > 1) {
        const long long tiles3 = 1LL * ((p.M + 63) / 64) * ((p.K + 63) / 64);
        if (8 * tiles3 <= n_cu) {
            best = 2;
            best_cost = static_cast<double>(64 * 128) / 0.72;   // one round of 64x128 at its table efficiency
        }
    }
    if (forced >= 0 && forced < GPULET_CONV_TILES) {
        best = forced;
        best_split = 1;
    }
    // The tall tile (224 pixels of one image x 128 filters, input patch in LDS) against the best
    // gathering tile, in the same units (tall_cost).
    int th11 = 0, tw11 = 0;
    double geo11 = 0.0;
    const bool tall_ok = tall_eligible(p, vec, &th11, &tw11, &geo11);
    if (forced < 0 && tall_ok && p.C >= 2 * BK) {
        const double cost = tall_cost(p, th11, tw11, geo11, n_cu);
        if (cost < best_cost) {
            best = 11;
            best_split = 1;
            best_cost = cost;
        }
    }
    int tw = 0;
    const bool patch_ok = patch_eligible(p, vec, &tw);
    if (best == 7 && !patch_ok) best = 1;  // the patch kernel does not apply: same tile shape, gathered
    // The patch kernel runs one workgroup per CU.  Measured on MI355X it beats the gathering
    // tiles whenever all of its workgroups are resident at once (a second round doubles its
    // time), from a single block of 64 channels on: 3x3 64 -> 64 on 56x56 at batch 8 5.5 against
    // 6.2 us, 128 -> 256 on 14x14 at batch 32 6.9 against 7.8, 192 -> 384 on 7x7 7.9 against 10.0.
    if (forced < 0 && patch_ok) {
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
    if (best == 11 && !tall_ok) best = 1;
    return Choice{best, best_split, tw, tw64, th11, tw11, (is_gathering_tile(best) || best == 11) ? best_cost : 0.0};
}

}  // namespace

hipError_t launch_conv(const ConvArgs &a, const LaunchCtx &ctx, hipStream_t stream) {
    ConvParams p;
    bool vec = false;
    const hipError_t st = make_params(a, ctx, p, vec);
    if (st != hipSuccess) return st;
    if (a.pre_pool) {
        // checked by check_conv: 3x3 window, 1x1 filter, stride 1, no padding, C % 8 == 0; the
        // callers check the 16-byte alignment of x and w
        if (!vec || p.ldx != a.C) return hipErrorInvalidValue;
        return launch_pooled_conv(p, stream);
    }

    if (a.post_pool2) {
        // the two kernels with a pooled epilogue: weights in registers for 64 input channels, else the tall tile
        int th = 0, tw = 0;
        double geo = 0.0;
        if (a.post_pool2 != 2 || a.y2 || a.pool_y) return hipErrorInvalidValue;
        if (c64_applicable(p, vec, &tw, true)) return launch_c64(p, tw, ctx.n_cu < 1 ? 1 : ctx.n_cu, true, stream);
        if (!tall_eligible(p, vec, &th, &tw, &geo, true)) return hipErrorInvalidValue;
        return launch_tall(p, th, tw, true, stream);
    }
    const Choice c = choose_kernel(p, vec, ctx);
    const int n_cu = ctx.n_cu < 1 ? 1 : ctx.n_cu;
    switch (c.best) {
        case 11: return launch_tall(p, c.th11, c.tw11, false, stream);
        case 10: return launch_c64(p, c.tw64, n_cu, false, stream);
        case 9: return launch_stem(p, n_cu, stream);
        case 8: return launch_stream(p, n_cu, stream);
        case 7: return launch_patch(p, c.tw, stream);
        default: {
            const long long tiles128 = 1LL * ((p.M + 127) / 128) * ((p.K + 127) / 128);
            return launch_igemm(p, vec, c.best, c.split, tiles128 > n_cu, stream);
        }
    }
}

// The pooled epilogue saves the layer's full-size store and the pool kernel's pass over it (at
// least a sixth of the pair's time on the layers it applies to), so the tall tile may cost up to
// 15 % more than the kernel the layer would get by itself.  Layers that a specialised kernel takes
// (all workgroups of the patch kernel resident, 64 input channels) keep it and their pool kernel.
bool conv_pool2_fusable(const ConvArgs &a, const LaunchCtx &ctx) {
    if (!g_pool_fusion.load() || g_tile_override.load() >= 0) return false;
    if (a.pre_pool || a.y2 || a.pool_y || a.residual || !a.relu) return false;
    ConvParams p;
    bool vec = false;
    if (make_params(a, ctx, p, vec) != hipSuccess) return false;
    int th = 0, tw = 0;
    double geo = 0.0;
    const Choice c = choose_kernel(p, vec, ctx);
    if (c.best == 10) return c64_applicable(p, vec, &tw, true);   // the same kernel with another epilogue
    if (p.C < 2 * BK || !tall_eligible(p, vec, &th, &tw, &geo, true)) return false;
    if (c.cost <= 0.0) return false;
    return tall_cost(p, th, tw, geo, ctx.n_cu < 1 ? 1 : ctx.n_cu) <= 1.15 * c.cost;
}

// Independent layers in one launch.  Every member must be a layer the gathering kernel would
// run anyway, unsplit: 16-byte gathers, no fused pool, one output, and none of the specialised
// kernels chosen for its shape; otherwise the members are launched one after the other.  The
// tile shared by all members minimises the work on the busiest CU over the members' tiles
// together.  Results are those of separate launches, bit for bit.
hipError_t launch_conv_group(const ConvArgs *a, int n, const LaunchCtx &ctx, hipStream_t stream, int *launches) {
    ConvParams p[MAX_GROUP];
    bool together = n >= 2 && n <= MAX_GROUP;
    const int forced = g_tile_override.load();
    for (int j = 0; j < n && together; ++j) {
        bool vec = false;
        if (make_params(a[j], ctx, p[j], vec) != hipSuccess || !vec || a[j].pre_pool || a[j].y2 || a[j].pool_y) {
            together = false;
            break;
        }
        const Choice c = choose_kernel(p[j], vec, ctx);
        if (!is_gathering_tile(c.best) || c.split > 1) together = false;
    }
    if (launches) *launches = together ? 1 : n;
    if (!together) {
        for (int j = 0; j < n; ++j) {
            const hipError_t st = launch_conv(a[j], ctx, stream);
            if (st != hipSuccess) return st;
        }
        return hipSuccess;
    }
    const int n_cu = ctx.n_cu < 1 ? 1 : ctx.n_cu;
    long long tiles128 = 0, slices128 = 0;
    for (int j = 0; j < n; ++j) {
        const long long tj = 1LL * ((p[j].M + 127) / 128) * ((p[j].K + 127) / 128);
        tiles128 += tj;
        slices128 += tj * ((p[j].Kg + BK - 1) / BK);
    }
    int best = 0;
    double best_cost = 0.0;
    for (int o = 0; o < kNumTiles; ++o) {
        const TileChoice &t = kTiles[o];
        long long tiles = 0;
        for (int j = 0; j < n; ++j) tiles += 1LL * ((p[j].M + t.bm - 1) / t.bm) * ((p[j].K + t.bn - 1) / t.bn);
        double eff = t.eff;
        // the same bonus as in a single launch for 128x128 with two workgroups per CU, at the
        // members' mean depth (inception 3a's group at batch 32: 18.0 -> 15.8 us)
        if (t.id == 0 && tiles128 > n_cu) eff = std::min(1.2, 0.90 + 3.0 * tiles128 / slices128);
        const double cost = static_cast<double>((tiles + n_cu - 1) / n_cu) * t.bm * t.bn / eff;
        if (o == 0 || cost < best_cost) {
            best = t.id;
            best_cost = cost;
        }
    }
    if (is_gathering_tile(forced)) best = forced;
    return launch_igemm_group(p, n, best, tiles128 > n_cu, stream);
}

void set_conv_split_k(int max_split) { g_max_split_k.store(max_split); }

void set_conv_pool_fusion(int on) { g_pool_fusion.store(on ? 1 : 0); }

void set_conv_tile(int tile) { g_tile_override.store(tile); }

}  // namespace gpulet
