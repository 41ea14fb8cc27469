/*
 * gpulet.h - C ABI of the MI355X-native hot path behind gpu-lets.
 *
 * Paper: "Multi-model Machine Learning Inference Serving with GPU Spatial
 * Partitioning" (arXiv 2109.01611).  A gpu-let is a virtual GPU holding p% of
 * one physical GPU's compute (Sec. 2.3); a batch of b requests of model m is
 * served on it with latency L(b, p) (Sec. 3.1, Fig. 3; Table 2), and at most
 * two gpu-lets share a GPU, their sizes summing to at most 100 (Sec. 1;
 * Sec. 4.3 "Split": p and 100-p).  Here a gpu-let is a CU-masked HIP stream,
 * and the forward pass (the paper's executors ran PyTorch's, Sec. 5) is a set
 * of hand-written gfx950 kernels.
 *
 * Conventions for every call
 *   - Returns a gpulet_status: 0 on success, negative on error.  Nothing
 *     throws or aborts.  After GPULET_EHIP, gpulet_last_hip_error() gives the
 *     hipError_t (per calling thread).
 *   - Tensor pointers are DEVICE pointers owned by the caller; the library
 *     never frees or keeps them past the call's enqueued work.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Kernel calls only enqueue work on it; they do not synchronise.
 *   - Layouts: activations NHWC bf16 (n, h, w, c with c fastest); convolution
 *     weights KRSC bf16 ([K][R][S][C]); FC weights [Out][In] bf16 with In in
 *     the NHWC flatten order of the tensor feeding it; bias fp32.
 *   - Arithmetic: bf16 x bf16 products accumulated in fp32 (MFMA), bias,
 *     residual and ReLU in fp32, one round-to-nearest-even to bf16 on store.
 */
#ifndef GPULET_H
#define GPULET_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t gpulet_status;

enum {
    GPULET_OK = 0,
    GPULET_EINVAL = -1,   /* NULL pointer, non-positive or overflowing shape, pct outside 1..100 */
    GPULET_EOVERSUB = -2, /* more than two live gpu-lets on a device, or sizes summing past 100 */
    GPULET_EHIP = -3,     /* a HIP runtime call failed; see gpulet_last_hip_error() */
    GPULET_ENOMEM = -4    /* caller-provided workspace or output array too small */
};

/* Static, human-readable name of a status code. */
const char *gpulet_status_string(gpulet_status s);

/* hipError_t of the last GPULET_EHIP on the calling thread (0 if none). */
int gpulet_last_hip_error(void);

/* ------------------------------------------------------------------------
 * gpu-let = spatial partition (Sec. 2.3; Sec. 4.3 "Split").
 * ------------------------------------------------------------------------ */

/*
 * CU mask of a gpu-let of `pct` percent on a device of n_cu_total compute
 * units in n_xcd equal dies.  Pure integer host code, no GPU needed.
 *
 * The paper gives sizes in percent; a CU mask needs a whole number of CUs.
 * Every die contributes the same count (workgroups are dealt round-robin to
 * the dies), and that count is a multiple of the 4 shader engines of a die
 * (workgroups are dealt round-robin to those as well, so the engine with the
 * fewest CUs in the mask sets the pace; CU c of a die is in engine c % 4):
 *   share(pct) = 4 * ((pct * cus_per_xcd + 200) / 400)   (integer division),
 * clamped to 4 .. cus_per_xcd - 4 for pct < 100 (share(100) = cus_per_xcd), so
 * a Split always leaves the partner a balanced share.  On 32 CUs per die the
 * paper's sizes 20/40/50/60/80 become 8/12/16/20/24 CUs per die (25, 37.5,
 * 50, 62.5, 75 % of the device).  Dies whose CU count is not a multiple of 4,
 * or below 8, round to whole CUs instead: (pct * cus_per_xcd + 50) / 100,
 * clamped to 1 .. cus_per_xcd - 1.  which = 0 takes
 * the first share(pct) CUs of every die; which = 1 is the partner produced by
 * Split: it takes what a which = 0 gpu-let of (100 - pct) leaves, i.e.
 * cus_per_xcd - share(100 - pct) CUs per die, so the two are disjoint and
 * together cover the device.
 *
 * Mask bit i names CU (i / n_xcd) of die (i % n_xcd): the driver deals mask
 * bits round-robin over the dies.
 *
 * words[]: at least (n_cu_total + 31) / 32 entries (n_words_cap says how
 * many); *n_words receives the count written, *n_cu the popcount.
 * Errors: GPULET_EINVAL (NULL, pct outside 1..100, which outside 0..1,
 * n_cu_total not a positive multiple of n_xcd, a share of zero CUs),
 * GPULET_ENOMEM (n_words_cap too small).
 */
gpulet_status gpulet_mask_for_pct(int n_cu_total, int n_xcd, int pct, int which,
                                  uint32_t *words, int n_words_cap, int *n_words, int *n_cu);

typedef struct gpulet_partition gpulet_partition; /* opaque, library-owned */

/*
 * Create a gpu-let of `pct` percent on HIP device `device`: computes the mask
 * as above from the device's CU count and creates a CU-masked stream.
 * At most two gpu-lets may be live per device and their pct must sum to at
 * most 100 (Sec. 1: up to two per GPU); otherwise GPULET_EOVERSUB.  Two live
 * gpu-lets must use different `which`.  *out is set only on success and must
 * be released with gpulet_partition_destroy.  Thread-safe.
 */
gpulet_status gpulet_partition_create(int device, int pct, int which, gpulet_partition **out);

/* Synchronises the stream, destroys it and frees the record.  Destroying a
 * handle twice, or NULL, returns GPULET_EINVAL. */
gpulet_status gpulet_partition_destroy(gpulet_partition *p);

/*
 * Facts of a live gpu-let.  Any output pointer may be NULL.  mask_words must
 * have room for 8 words (256 CUs); *n_words says how many are meaningful.
 * *hip_stream is the hipStream_t to pass as `stream` below.
 */
gpulet_status gpulet_partition_info(const gpulet_partition *p, int *device, int *pct, int *which,
                                    int *n_cu, int *n_cu_total, uint32_t mask_words[8],
                                    int *n_words, void **hip_stream);

/* Mask the HIP runtime reports for the gpu-let's stream (hipExtStreamGetCUMask);
 * same array rules as above. */
gpulet_status gpulet_partition_query_mask(const gpulet_partition *p, uint32_t mask_words[8],
                                          int *n_words);

/* Request bookkeeping (Sec. 5: the frontend forms batches and dispatches each
 * to the executor of one gpu-let): batches and images run on this gpu-let
 * through gpulet_run_model and the profiling calls, exact integers. */
gpulet_status gpulet_partition_counters(const gpulet_partition *p, uint64_t *batches_run,
                                        uint64_t *images_run);

/* Kernel launches enqueued on this gpu-let by gpulet_run_model, gpulet_profile_model
 * and gpulet_profile_corun since it was created (layers that share a launch count
 * once; graph replays launch no kernels from the host and are not counted).  Lets a
 * profiler attribute per-dispatch counters to batches. */
gpulet_status gpulet_partition_kernel_launches(const gpulet_partition *p, uint64_t *launches);

/* Blocks until all work enqueued on the gpu-let's stream has finished. */
gpulet_status gpulet_partition_sync(gpulet_partition *p);

/*
 * Runs n_blocks workgroups of a tiny kernel on the gpu-let and records, per
 * workgroup, where the hardware placed it: out[2*i] = die (XCC) id,
 * out[2*i+1] = the hardware id register (shader engine, shader array and CU
 * fields).  `out` is a DEVICE array of 2*n_blocks uint32.  Synchronises.
 * Used to check that a mask is honoured and which physical CUs it names.
 */
gpulet_status gpulet_partition_probe(gpulet_partition *p, uint32_t *out, int n_blocks);

/*
 * Measurement aid for the roofline of the convolution kernels (the matrix-core
 * utilisation asked of the per-partition profile, paper Sec. 3.1): runs one
 * workgroup of waves_per_cu (4 or 8) wavefronts per CU of the gpu-let, each
 * issuing 64 * iters 32x32x16 bf16 matrix instructions on register operands and
 * nothing else, `launches` times back to back between one event pair (after
 * one untimed launch).  dense != 0: pseudo-random operands in (-1, 1);
 * dense == 0: all-zero operands.  *avg_ms = milliseconds per launch,
 * *tflops = the rate.  The difference between the two patterns is the engine
 * clock the power limit allows.  Uses the gpu-let's scratch for the kernel's
 * (meaningless) output.  Synchronises.  GPULET_EINVAL for other wave counts or
 * counts below 1.
 */
gpulet_status gpulet_partition_mfma_rate(gpulet_partition *p, int dense, int waves_per_cu, int iters,
                                         int launches, float *avg_ms, double *tflops);

/* The same probe, launched through a captured HIP graph when via_graph != 0:
 * checks that graph replays on a gpu-let's stream honour its CU mask too. */
gpulet_status gpulet_partition_probe_ex(gpulet_partition *p, uint32_t *out, int n_blocks,
                                        int via_graph);

/* ------------------------------------------------------------------------
 * Layers of the forward pass (Sec. 5; models of Table 4).
 * ------------------------------------------------------------------------ */

/*
 * Convolution layer, implicit GEMM on MFMA with fused bias and ReLU:
 *   y[n,p,q,k] = act(b[k] + sum_{r,s,c} x[n, p*stride-pad+r, q*stride-pad+s, c] * w[k,r,s,c])
 * with x taken as zero outside the image (cross-correlation, no kernel flip)
 * and P = (H + 2*pad - R) / stride + 1, Q likewise from W and S.
 * x: N*H*W*C bf16, w: K*R*S*C bf16, b: K fp32 (NULL = no bias), y: N*P*Q*K bf16.
 * Errors: GPULET_EINVAL for NULL x/w/y, non-positive sizes, pad < 0, empty
 * output, or any tensor of 2^30 or more elements (byte offsets are 32-bit).
 */
gpulet_status gpulet_conv2d_fwd(const void *x, const void *w, const float *b, void *y, int N,
                                int C, int H, int W, int K, int R, int S, int stride, int pad,
                                int relu, void *stream);

/*
 * Same, plus what residual and inception blocks need:
 *   residual      NULL, or a bf16 tensor N*P*Q*K (dense) added before the ReLU;
 *   y_ch_stride   channels per pixel of the tensor y points into (0 means K);
 *   y_ch_offset   first channel written, so a branch lands directly inside a
 *                 concatenated tensor: y[((n*P+p)*Q+q)*y_ch_stride + y_ch_offset + k].
 * Extra error: y_ch_offset < 0 or y_ch_offset + K > y_ch_stride.
 */
gpulet_status gpulet_conv2d_fwd_ex(const void *x, const void *w, const float *b, void *y, int N,
                                   int C, int H, int W, int K, int R, int S, int stride, int pad,
                                   int relu, const void *residual, int y_ch_stride,
                                   int y_ch_offset, void *stream);

/*
 * Same as gpulet_conv2d_fwd_ex for an input that is a channel slice of a wider
 * tensor: the layer reads x[((n*H+h)*W+w)*x_ch_stride + x_ch_offset + c] for
 * c < C (x_ch_stride 0 means C).  Used when several layers that read the same
 * tensor are computed as one layer and their consumers each take a slice of the
 * result (the two reduce layers of an inception block).  Only the gathering
 * tiles 0..6 read slices; another forced tile falls back as documented at
 * gpulet_set_conv_tile.  Results have the bits of the same layer on a dense copy
 * of the slice.  Extra error: x_ch_offset < 0 or x_ch_offset + C > x_ch_stride.
 */
gpulet_status gpulet_conv2d_fwd_slices(const void *x, const void *w, const float *b, void *y, int N,
                                       int C, int H, int W, int K, int R, int S, int stride, int pad,
                                       int relu, const void *residual, int x_ch_stride, int x_ch_offset,
                                       int y_ch_stride, int y_ch_offset, void *stream);

/*
 * A 1x1 convolution (pad 0) whose filters are stored to two tensors: filters
 * [0, k2) to y and filters [k2, K) to y2, each optionally as a channel slice of
 * wider pixels (y_ch_stride / y_ch_offset and y2_ch_stride / y2_ch_offset, 0 =
 * dense), the input optionally a slice too (as gpulet_conv2d_fwd_slices).  One
 * launch then serves layers that read the same tensor but whose results live in
 * different places: in an inception block the 1x1 branch, which belongs to the
 * concatenated output, and the two reduce layers, whose result feeds the 3x3 and
 * 5x5 layers.  w: K*C bf16 and b: K fp32 hold the filters of both parts in order.
 * Each output element has the bits gpulet_conv2d_fwd_ex gives for its filter.
 * Errors: those of gpulet_conv2d_fwd_ex; GPULET_EINVAL unless 0 < k2 < K and
 * y2 is not NULL, or when a slice does not fit its pixels; C must be a multiple
 * of 8 and x, w 16-byte aligned (GPULET_EINVAL otherwise).
 */
gpulet_status gpulet_conv1x1_fwd_two_outputs(const void *x, const void *w, const float *b, void *y,
                                             void *y2, int N, int C, int H, int W, int K, int k2,
                                             int stride, int relu, int x_ch_stride, int x_ch_offset,
                                             int y_ch_stride, int y_ch_offset, int y2_ch_stride,
                                             int y2_ch_offset, void *stream);

/*
 * Up to 4 independent convolution layers in ONE launch: the workgroups of all
 * layers form one grid, so small layers that do not depend on one another (the
 * 3x3, 5x5 and pooling-branch layers of an inception block; a projection
 * shortcut and the first layer of its residual block) pay the fixed cost of a
 * launch once and fill the GPU together.  Each member is described as for
 * gpulet_conv2d_fwd_slices.  Members must not read (x, residual) or overwrite
 * memory another member writes; channel slices of one tensor (same y, same
 * y_ch_stride, disjoint channels) count as different destinations.  Each
 * member's result has the bits of its own gpulet_conv2d_fwd_slices call.  When a
 * member cannot share (channel count not a multiple of 8, misaligned operands,
 * or a shape for which a specialised kernel is chosen) the members are launched
 * one after the other on `stream` instead: same results.
 * Errors: GPULET_EINVAL for n outside 1..4, a member that gpulet_conv2d_fwd_slices
 * would reject, or members that depend on one another.
 */
typedef struct gpulet_conv_desc {
    const void *x, *w;
    const float *b;
    void *y;
    const void *residual;
    int32_t N, C, H, W, K, R, S, stride, pad, relu;
    int32_t x_ch_stride, x_ch_offset, y_ch_stride, y_ch_offset;
} gpulet_conv_desc;
gpulet_status gpulet_conv2d_group_fwd(const gpulet_conv_desc *layers, int n, void *stream);

/*
 * A 1x1 convolution (pad 0, stride 1) that also writes, from the same launch,
 * pool_y = maxpool(x, window 3x3, stride 1, pad 1) (N*H*W*C bf16, maximum over
 * in-image taps only, the bits of gpulet_pool): extra workgroups at the end of
 * the convolution's grid do the pooling, so the pool costs no launch of its own.
 * In an inception block the pool of the block's input feeds the pooling branch
 * while the 1x1 layers read the same input.  y2 may be NULL (one output, k2
 * ignored) or, as in gpulet_conv1x1_fwd_two_outputs, receive filters [k2, K).
 * x must be dense (no input slice).  Errors as gpulet_conv1x1_fwd_two_outputs,
 * and GPULET_EINVAL for a NULL or misaligned pool_y.
 */
gpulet_status gpulet_conv1x1_maxpool3_fwd(const void *x, const void *w, const float *b, void *y, void *y2,
                                          void *pool_y, int N, int C, int H, int W, int K, int k2,
                                          int relu, int y_ch_stride, int y_ch_offset, int y2_ch_stride,
                                          int y2_ch_offset, void *stream);

/*
 * A 3x3 / stride 1 / pad 1 convolution with ReLU and the 2x2 / stride 2 max pool
 * behind it (the end of every VGG-16 group, Table 4) in one kernel:
 *   y = maxpool2x2(relu(b + conv3x3(x, w)))
 * The layer's own output is never written: the kernel's epilogue takes the
 * maximum of each 2x2 window of a tile's fp32 sums, then adds the bias, applies
 * the ReLU and rounds once (rounding and ReLU do not decrease, so for finite
 * sums the result has the bits of gpulet_conv2d_fwd_ex followed by gpulet_pool;
 * a NaN sum loses against any number here, while the pool kernel orders NaN
 * bit patterns like numbers).  x: N*H*W*C
 * bf16, w: K*3*3*C bf16, b: K fp32 or NULL, y: N*(H/2)*(W/2) pixels of
 * y_ch_stride channels (0 = K), filter k stored at channel y_ch_offset + k.
 * Device pointers owned by the caller; asynchronous on `stream`.
 * GPULET_EINVAL unless H and W are even, C is a multiple of 64, K, y_ch_stride
 * and y_ch_offset are multiples of 8 and x, w, b, y are 16-byte aligned; other
 * errors as gpulet_conv2d_fwd_ex.
 */
gpulet_status gpulet_conv3x3_maxpool2_fwd(const void *x, const void *w, const float *b, void *y, int N, int C,
                                          int H, int W, int K, int y_ch_stride, int y_ch_offset, void *stream);

/*
 * Whether gpulet_run_model and its relatives (profile, co-run, graph capture) may
 * run a convolution and the 2x2 / stride 2 max pool that follows it as one launch
 * (1, the default) or always as two kernels (0).  When allowed, a pair is fused
 * per launch if the pool is the only reader of the layer's output, the layer
 * qualifies for gpulet_conv3x3_maxpool2_fwd and either runs the kernel that
 * keeps the weights of 64 input channels in registers anyway (that kernel pools
 * in its epilogue when its column blocks are a power of two wide) or has at
 * least 128 input channels and the tall-tile kernel, which pools in its
 * epilogue, costs the layer at most 15 % more than the kernel it would run
 * otherwise; the layer's own output buffer is then left unwritten.  Results are
 * bit-identical either way.  Process-wide.
 */
gpulet_status gpulet_set_conv_pool_fusion(int on);

/*
 * Pooling branch of an inception block (GoogLeNet of Table 4) in one kernel:
 *   y = act(b + conv1x1(maxpool(x, window 3x3, stride 1, pad 1), w))
 * with the pool's maximum taken over in-image taps only, as in gpulet_pool.
 * The pooled tensor is never written; the result has the bits of gpulet_pool
 * followed by gpulet_conv2d_fwd_ex.  x: N*H*W*C bf16, w: K*C bf16, b: K fp32
 * or NULL, y and the channel-slice arguments as in gpulet_conv2d_fwd_ex.
 * Errors: those of gpulet_conv2d_fwd_ex, and GPULET_EINVAL unless C is a
 * multiple of 8 and x and w are 16-byte aligned.
 */
gpulet_status gpulet_maxpool3_conv1x1_fwd(const void *x, const void *w, const float *b, void *y, int N,
                                          int C, int H, int W, int K, int relu, int y_ch_stride,
                                          int y_ch_offset, void *stream);

/*
 * Measurement aid for the time decomposition of a convolution launch (the
 * per-partition latency profile of Sec. 3.1 is made of such launches): runs the
 * layer `warmup` times as gpulet_conv2d_fwd would, then once more with the
 * kernel's first workgroups (at most 8) recording the device's wall clock (a
 * constant 100 MHz counter shared by the whole GPU: 10 ns units) at these
 * points of their life:
 *   0 first instruction            1 argument block fetched, tile decoded
 *   2 position table complete      3 first input patch and weights in LDS
 *   4 end of the main loop         5 fp32 tile staged in LDS
 *   6 output stores issued         7 unused (0)
 * (tiles 7 and 11 of gpulet_set_conv_tile).  The kernel that keeps the weights
 * of 64 input channels in registers (tile 10) walks over many pixel tiles and
 * records instead: 0 first instruction, 1 weights requested, and around its
 * fourth pixel tile 2 arrival at the "patch landed" barrier, 3 patch there,
 * 4 matrix instructions issued, 5 patch released, 6 output stores issued,
 * 7 arrival at the next tile's barrier (7 - 2 = one tile period).
 * stamps: HOST array of 8 x 8 int64, row = workgroup; *workgroups = how many
 * rows were filled: 0 when the kernel that runs this layer records no stamps
 * (the gathering, streaming, stem and depthwise kernels).  Allocates and frees a 512-byte device buffer;
 * synchronises.  Errors as gpulet_conv2d_fwd; GPULET_EINVAL for NULL stamps or
 * workgroups or a negative warmup.
 */
gpulet_status gpulet_conv2d_timeline(const void *x, const void *w, const float *b, void *y, int N, int C,
                                     int H, int W, int K, int R, int S, int stride, int pad, int relu,
                                     void *stream, int warmup, int64_t *stamps, int *workgroups);

/*
 * Tuning and testing knob: force every later convolution launch of the
 * process onto one workgroup tile (pixels x channels):
 *   0: 128x128  1: 128x64  2: 64x128  3: 64x64  4: 128x32  5: 32x128  6: 256x128
 *   7: 128x64 with the input patch of a tile resident in LDS (3x3 filters,
 *      stride 1, pad 1, C a multiple of 64; other shapes run tile 1 instead)
 *   8: 64x128 walked by workgroups that keep their weights in LDS and stream
 *      over many pixel tiles (1x1 filters, C a multiple of 8 up to 128; other shapes run
 *      tile 2 instead)
 *   9: 4 rows x 32 columns of one image by 32 or 64 channels, for inputs of at
 *      most 4 channels (image stems): the tile's input patch sits in LDS as
 *      4-channel pixels and filter rows are padded to 16 or 32 elements
 *      (filters of 3, 5 or 7 rows and at most 8 columns; other shapes run
 *      tile 1 instead)
 *  10: 128x64 walked by workgroups that keep their 64 filters' weights in
 *      registers (3x3 filters, stride 1, pad 1, exactly 64 input channels, no
 *      residual operand; other shapes run tile 1 instead)
 *  11: 224x128: a rectangle of up to 224 pixels of one image (8 x 28 on maps
 *      56, 112 or 224 pixels wide) with its input patch resident in LDS and
 *      the weights streamed one filter tap at a time (3x3 filters, stride 1,
 *      pad 1, C a multiple of 64; other shapes run tile 1 instead)
 *  12: 192x128  13: 96x128 (gathering tiles with three 32-pixel row tiles per
 *      wavefront, for layers whose 128-pixel tiles just miss a whole number of
 *      rounds on a gpu-let),
 * or -1 to return to automatic selection, which picks the tile whose busiest
 * CU has the least work for the launch's shape and the stream's CU count, and
 * tile 9 wherever it applies.  All tiles but 9 give bit-identical results; tile 9
 * groups the same ascending sum differently (zero padding inside the depth),
 * so it agrees with them to rounding.  Tiles 7..11 need dense input pixels and
 * a single output: a layer that reads a channel slice or stores to two tensors
 * counts as another shape for them.  GPULET_EINVAL outside -1..13.
 */
enum { GPULET_CONV_TILES = 14 };
gpulet_status gpulet_set_conv_tile(int tile);

/*
 * Largest number of workgroups that may share one output tile by splitting the
 * depth (1..8; default 1 = splitting off).  When allowed, splitting is used on a
 * gpu-let's stream when a layer has too few tiles for the gpu-let's CUs; partial
 * tiles meet in scratch memory owned by the gpu-let and are summed in fp32 in a
 * fixed order, so results are reproducible run to run, but they differ in the
 * last bits from the unsplit sum.  With splitting off, an image's result does
 * not depend on the batch it is part of or on the gpu-let's size.  A forced tile
 * (gpulet_set_conv_tile) never splits.  Launches on streams that do not belong
 * to a gpu-let never split.
 */
gpulet_status gpulet_set_conv_split_k(int max_split);

/*
 * Depthwise convolution (one R x S filter per channel; the depthwise-separable
 * blocks of the SSD-MobileNet of Table 4), fused bias and ReLU:
 *   y[n,p,q,c] = act(b[c] + sum_{r,s} x[n, p*stride-pad+r, q*stride-pad+s, c] * w[r,s,c])
 * x: N*H*W*C bf16 NHWC, w: R*S*C bf16 (channel fastest), b: C fp32 or NULL,
 * y: N*P*Q*C bf16.  fp32 accumulation in (r, s) order, one rounding to bf16.
 * Bound by memory traffic (one multiply-add per input element), so it runs on
 * the vector units.  GPULET_EINVAL for NULL x/w/y, non-positive sizes, an
 * empty output or tensors of 2^30 elements or more.
 */
gpulet_status gpulet_depthwise_conv2d_fwd(const void *x, const void *w, const float *b, void *y, int N, int C,
                                          int H, int W, int R, int S, int stride, int pad, int relu,
                                          void *stream);

enum { GPULET_POOL_MAX = 0, GPULET_POOL_AVG = 1, GPULET_POOL_GLOBAL_AVG = 2 };

/*
 * Pooling over NHWC bf16.  mode MAX: maximum over the in-image taps of a
 * k x k window (padding never wins).  mode AVG: sum of the in-image taps
 * divided by k*k (padding counts as zero).  mode GLOBAL_AVG: mean over the
 * H x W plane (k, stride, pad ignored), output N*1*1*C.  Sums are fp32.
 * Output extent as for convolution.  Requires pad < k.
 */
gpulet_status gpulet_pool(const void *x, void *y, int N, int C, int H, int W, int mode, int k,
                          int stride, int pad, void *stream);

/*
 * Fully connected layer on MFMA:
 *   y[n,o] = act(b[o] + sum_i x[n,i] * w[o,i])
 * x: N*In bf16, w: Out*In bf16, b: Out fp32 or NULL, y: N*Out, bf16 or (if
 * out_fp32) fp32.
 */
gpulet_status gpulet_fc(const void *x, const void *w, const float *b, void *y, int N, int In,
                        int Out, int relu, int out_fp32, void *stream);

/*
 * gpulet_fc for callers that cannot allocate device memory (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): same
 * arguments, same result, bit for bit, as gpulet_fc on the same stream, but
 * the partial tiles and arrival counters that long rows (In >= 8192, N <= 32)
 * split over several workgroups need live in an array that is part of the
 * library's device image (2 MiB of tiles + 1024 counters per GPU, held until
 * the process ends) instead of a gpu-let's allocation.  The call allocates and
 * frees nothing, on the host's HIP side or the device.  x, w, b, y are device
 * pointers owned by the caller; the call is asynchronous on `stream` (a
 * gpu-let's stream sizes the split from the gpu-let's CU count, any other
 * stream from the device's).
 * Limit: ceil(Out/64) * ksplit * (N <= 16 ? 4 : 8) KiB <= 2 MiB and
 * ceil(Out/64) <= 1024, with ksplit = min(8, CUs / ceil(Out/64)) when that is
 * at least 2; a layer beyond it returns GPULET_ENOMEM and launches nothing.
 * Layers that need no scratch (short rows, N > 32, a single depth range) are
 * never refused.  Other errors as gpulet_fc.
 * All calls on one GPU share the array: calls that overlap in time on one GPU
 * (two streams, two threads) race and give undefined results; calls ordered on
 * one stream do not.  The counters are cleared by a small kernel on `stream`
 * before each use, so a call does not depend on what an earlier one left.
 */
gpulet_status gpulet_fc_static_scratch(const void *x, const void *w, const float *b, void *y, int N, int In,
                                       int Out, int relu, int out_fp32, void *stream);

/* ------------------------------------------------------------------------
 * Whole model on a gpu-let (Sec. 5 "Backend inference executor").
 * ------------------------------------------------------------------------ */

enum { GPULET_OP_CONV = 0, GPULET_OP_POOL = 1, GPULET_OP_FC = 2, GPULET_OP_DWCONV = 3 };

/*
 * One layer.  Activations live in numbered buffers; a layer reads in_buf and
 * writes out_buf.  Spatial sizes are inferred by the library from the model
 * input.  Fields not used by an op are ignored.
 */
typedef struct gpulet_layer {
    int32_t op;            /* GPULET_OP_* */
    int32_t in_buf;        /* buffer read */
    int32_t out_buf;       /* buffer written */
    int32_t res_buf;       /* CONV: buffer added before the ReLU, or -1 */
    int32_t C;             /* CONV/DWCONV/POOL: input channels; FC: In (= C*H*W of in_buf) */
    int32_t K;             /* CONV: output channels; FC: Out */
    int32_t R;             /* CONV/DWCONV: kernel height; POOL: window k */
    int32_t S;             /* CONV/DWCONV: kernel width */
    int32_t stride;
    int32_t pad;
    int32_t relu;          /* CONV/DWCONV/FC */
    int32_t mode;          /* POOL: GPULET_POOL_* */
    int32_t out_ch_total;  /* CONV: channels of out_buf when this layer writes a slice of
                              a concatenated tensor; 0 means K */
    int32_t out_ch_offset; /* CONV: first channel written */
    int32_t out_fp32;      /* FC: store fp32 instead of bf16 */
    int32_t pre_pool;      /* CONV: 0, or 3 = a 3x3 / stride 1 / pad 1 max pool of in_buf comes first
                              (gpulet_maxpool3_conv1x1_fwd; 1x1 filters, stride 1, pad 0, C % 8 == 0) */
    int32_t in_ch_total;   /* CONV: channels of in_buf when this layer reads only C of them (the
                              output of several layers computed as one); 0 means C */
    int32_t in_ch_offset;  /* CONV: first channel read */
    int32_t K2;            /* CONV, 1x1 filters without residual: when > 0 the last K2 of the K filters are
                              stored to out2_buf and only the first K - K2 to out_buf (several layers
                              that read one tensor computed as one; see gpulet_conv1x1_fwd_two_outputs) */
    int32_t out2_buf;      /* CONV with K2 > 0: second buffer written */
    int32_t out2_ch_total; /* CONV with K2 > 0: channels of out2_buf when a slice is written; 0 means K2 */
    int32_t out2_ch_offset;/* CONV with K2 > 0: first channel written in out2_buf */
    int32_t side_pool;     /* CONV, 1x1 filters, pad 0, C % 8 == 0, dense input: 0, or 3 = the launch also
                              writes the 3x3 / stride 1 / pad 1 max pool of in_buf to pool_buf
                              (gpulet_conv1x1_maxpool3_fwd) */
    int32_t pool_buf;      /* CONV with side_pool: buffer that receives the pooled tensor */
    int32_t group_next;    /* CONV: 1 = the next layer (a CONV too) is independent of this one and may
                              share its launch (gpulet_conv2d_group_fwd); chains of up to 4 layers */
    const void *w;         /* device: CONV KRSC bf16, DWCONV RSC bf16, FC [Out][In] bf16 */
    const float *b;        /* device: fp32 bias or NULL */
} gpulet_layer;

/*
 * A model: layers in execution order over n_bufs buffers.  Buffer in_buf is
 * the caller's input tensor (N, in_H, in_W, in_C), buffer out_buf the caller's
 * output; all others are carved from the workspace.  A buffer may be written
 * by several layers (disjoint channel slices, or reuse after its readers have
 * run); its size is the largest it ever needs.  Every buffer must be written
 * before it is read.
 */
typedef struct gpulet_model_desc {
    int32_t n_layers;
    int32_t n_bufs;
    int32_t in_C, in_H, in_W;
    int32_t in_buf;
    int32_t out_buf;
    int32_t reserved;
    const gpulet_layer *layers;
} gpulet_model_desc;

/*
 * Number of streams ("lanes", all with the gpu-let's CU mask) the model runner
 * spreads independent layers over (inception branches, a projection shortcut
 * next to the main path, detection heads).  Only 1 is accepted at present:
 * every layer runs on the gpu-let's stream in table order.  A second lane is
 * implemented (dependencies through buffers, reused ones included, become
 * event waits; see gpulet_model_schedule) but switched off; GPULET_EINVAL for
 * any other value.
 */
gpulet_status gpulet_set_model_lanes(int lanes);

/*
 * How the model runner would spread `m` over `lanes` lanes (1..2; host only,
 * nothing is launched): lane[i] for each of the n_layers layers, and the
 * cross-lane waits as pairs (wait_from[k] must complete before wait_to[k]
 * starts).  Layers of one lane run in table order.  GPULET_ENOMEM if there are
 * more than max_waits pairs (*n_waits then holds the number).
 */
gpulet_status gpulet_model_schedule(const gpulet_model_desc *m, int batch, int lanes, int *lane,
                                    int *wait_from, int *wait_to, int max_waits, int *n_waits);

/* Bytes of workspace gpulet_run_model needs for `batch` images (a multiple of
 * 256).  GPULET_EINVAL if the description is inconsistent (channel or feature
 * counts that do not match the inferred shapes, bad buffer indices, a buffer
 * read before written, empty outputs). */
gpulet_status gpulet_model_workspace_bytes(const gpulet_model_desc *m, int batch, size_t *bytes);

/* Inferred shape of one buffer for one image (its last writer's view), its
 * element size in bytes, and its byte offset inside the workspace for `batch`
 * images (offset is (size_t)-1 for the model's input and output buffers). */
gpulet_status gpulet_model_buffer_info(const gpulet_model_desc *m, int batch, int buf, int *C,
                                       int *H, int *W, int *elem_bytes, size_t *ws_offset);

/*
 * Forward pass of one batch on a gpu-let: every layer is enqueued on the
 * partition's stream with no host synchronisation in between.  `in` is the
 * input batch (batch*in_H*in_W*in_C bf16), `out` receives the output buffer.
 * `workspace` must be 256-byte aligned device memory of at least
 * gpulet_model_workspace_bytes() bytes (GPULET_ENOMEM otherwise).
 * If latency_ms is not NULL the call brackets the batch with events, waits
 * for it and stores the elapsed milliseconds; if NULL it returns right after
 * enqueueing.  Counts one batch and `batch` images on the partition.
 */
gpulet_status gpulet_run_model(const gpulet_model_desc *m, int batch, gpulet_partition *p,
                               const void *in, void *out, void *workspace,
                               size_t workspace_bytes, float *latency_ms);

/*
 * The same forward pass as a HIP graph: all layers of one batch are captured
 * once on the gpu-let's stream and replayed with a single launch, which takes
 * the per-layer host launch cost off the latency of small batches (Sec. 3.1:
 * small batches cannot use the whole GPU; here they are launch bound too).
 * The graph is bound to the pointers, batch size and gpu-let given at creation;
 * the caller keeps all of them alive and unchanged until the graph is
 * destroyed, and destroys the graph before its gpu-let.
 */
typedef struct gpulet_graph gpulet_graph; /* opaque, library-owned */

/* Captures and instantiates the graph.  Errors as gpulet_run_model.  *out is set
 * only on success.  Must not be called while another thread is capturing. */
gpulet_status gpulet_model_graph_create(const gpulet_model_desc *m, int batch, gpulet_partition *p,
                                        const void *in, void *out_buf, void *workspace,
                                        size_t workspace_bytes, gpulet_graph **out);

/* Replays the graph once on its gpu-let's stream.  latency_ms as in
 * gpulet_run_model (NULL: enqueue only).  Counts one batch on the gpu-let. */
gpulet_status gpulet_model_graph_launch(gpulet_graph *g, float *latency_ms);

/* Replays the graph `warmup` + `iters` times, each timed replay bracketed by its
 * own event pair and waited for (one batch in flight), latencies as in
 * gpulet_profile_model.  total_ms may be NULL. */
gpulet_status gpulet_model_graph_profile(gpulet_graph *g, int warmup, int iters, float *latency_ms,
                                         float *total_ms);

/* Waits for the gpu-let's stream, then frees the graph.  NULL or an unknown
 * handle returns GPULET_EINVAL. */
gpulet_status gpulet_model_graph_destroy(gpulet_graph *g);

/* ------------------------------------------------------------------------
 * Profiling: the L(b, p) table and co-run interference (Sec. 3.1, 3.2, 4.1).
 * ------------------------------------------------------------------------ */

/*
 * Runs `warmup` untimed batches, then `iters` batches each bracketed by its
 * own event pair on the gpu-let's stream; latency_ms[i] receives batch i's
 * elapsed milliseconds.  With sync_each != 0 the host waits for a batch to
 * finish before dispatching the next (the serving pattern: one batch in
 * flight per gpu-let); with sync_each == 0 batches are enqueued back to back.
 * If total_ms is not NULL it receives the time from the first timed batch's
 * start to the last one's end.  Synchronises before returning.
 * sync_each == 2 is the throughput pass for batches of a few microseconds,
 * where an event record between two batches is itself a measurable part of the
 * time: one event pair around all `iters` batches, nothing in between;
 * total_ms (required) receives their time and latency_ms may be NULL (if not,
 * every entry receives total_ms / iters).
 */
gpulet_status gpulet_profile_model(const gpulet_model_desc *m, int batch, gpulet_partition *p,
                                   const void *in, void *out, void *workspace,
                                   size_t workspace_bytes, int warmup, int iters, int sync_each,
                                   float *latency_ms, float *total_ms);

/*
 * Two gpu-lets at once (Sec. 3.2): model A on partition pa and model B on pb
 * are driven by two host threads, each dispatching one batch at a time (timed
 * by its own event pair, waited for before the next) until `window_ms` of wall
 * time has passed after `warmup` untimed batches each; the timed windows of
 * the two threads start together.  The side whose window ends first stops;
 * the other stops after the batch it is running then, and that batch, which ran
 * partly alone, is not reported (it still counts in the gpu-let's counters), so
 * every reported latency is a co-run latency.  lat_a/lat_b (capacity cap_a/cap_b)
 * receive the per-batch latencies, *n_a and *n_b how many were recorded (batches
 * beyond the capacity still run but are not recorded).  pa and pb must be
 * different live gpu-lets of one device.
 */
gpulet_status gpulet_profile_corun(const gpulet_model_desc *ma, int batch_a, gpulet_partition *pa,
                                   const void *in_a, void *out_a, void *ws_a, size_t ws_a_bytes,
                                   const gpulet_model_desc *mb, int batch_b, gpulet_partition *pb,
                                   const void *in_b, void *out_b, void *ws_b, size_t ws_b_bytes,
                                   int warmup, double window_ms, float *lat_a, int cap_a,
                                   int *n_a, float *lat_b, int cap_b, int *n_b);

/* Mean, median and nearest-rank 99th percentile of n latencies (host, fp64).
 * The p-th percentile is the value at rank ceil(p/100 * n) of the sorted list. */
gpulet_status gpulet_latency_stats(const float *latency_ms, int n, double *mean, double *p50,
                                   double *p99);

/*
 * Times `iters` back-to-back launches of one convolution layer between a
 * single event pair on `stream` (after `warmup` untimed launches) and stores
 * the average milliseconds per launch.  Arguments as gpulet_conv2d_fwd_ex.
 * Synchronises.
 */
gpulet_status gpulet_time_conv2d(const void *x, const void *w, const float *b, void *y, int N,
                                 int C, int H, int W, int K, int R, int S, int stride, int pad,
                                 int relu, const void *residual, int y_ch_stride,
                                 int y_ch_offset, void *stream, int warmup, int iters,
                                 float *avg_ms);

#ifdef __cplusplus
}
#endif
#endif /* GPULET_H */
