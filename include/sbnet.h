/*
 * sbnet.h -- C ABI of the MI355X (gfx950) tiled sparse convolution library.
 *
 * The calls follow the problem statement of "SBNet: Sparse Blocks Network for Fast
 * Inference" (arXiv 1801.02108): a binary computation mask is reduced to a list of active
 * blocks (Sec. 3.1), overlapping input tiles are gathered into a dense stack (Sec. 3.2),
 * a regular unpadded convolution -- or a whole residual unit (Sec. 3.3) -- runs on the
 * stack, and the results are scattered or scatter-added back (Sec. 3.2, Sec. 3.4).
 *
 * Conventions shared by every call
 *  - All tensor pointers are DEVICE pointers unless a comment says "host".  The caller owns
 *    every buffer; the library allocates nothing and keeps no pointer after a call returns.
 *  - Feature maps are dense NHWC; tile stacks are [cap][tile_h][tile_w][C]; the element
 *    type is given by an sbnet_dtype.  Base pointers must be 16-byte aligned.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *    enqueue work; they never synchronise, except sbnet_read_count.
 *  - The number of active blocks lives on the device: `count` points to one int32 written
 *    by sbnet_reduce_mask.  Later calls read it on the device and process
 *    min(*count, cap) blocks, so no host round trip is needed between the steps.
 *  - `indices` is int32 [cap][3] = (n, by, bx): sample and block-grid coordinates, in
 *    lexicographic order.  Pixel origins follow from an sbnet_geom.
 *  - Return value: SBNET_OK, or an error detected on the host before anything is enqueued
 *    (bad argument, unsupported combination) or reported by the HIP runtime at launch.
 *    sbnet_last_error() gives a thread-local description of the last failure.
 */
#ifndef SBNET_H
#define SBNET_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SBNET_OK = 0,
    SBNET_EINVAL = 1,       /* null pointer, non-positive size, inconsistent geometry      */
    SBNET_ECAP = 2,         /* more active blocks than `cap` (sbnet_read_count only)       */
    SBNET_EUNSUPPORTED = 3, /* valid request the library has no kernel for                 */
    SBNET_EHIP = 4          /* the HIP runtime reported an error                           */
} sbnet_status;

typedef enum { SBNET_F32 = 0, SBNET_BF16 = 1, SBNET_F16 = 2, SBNET_U8 = 3 } sbnet_dtype;
typedef enum { SBNET_POOL_MAX = 0, SBNET_POOL_AVG = 1 } sbnet_pool;

/*
 * Block geometry in pixels of the tensor an operation touches (Sec. 3.1, Fig. 3).  Block
 * (by, bx) covers rows [boffset_h + by*bstride_h, +bsize_h) and the analogous columns.
 * Input side of a k x k, stride-s, SAME convolution with bo x bo output blocks:
 * bsize = (bo-1)*s + k, bstride = bo*s, boffset = -(k-1)/2 (tiles overlap by k - s).
 * Output side: bsize = bstride = bo, boffset = 0 (blocks do not overlap).
 */
typedef struct {
    int bsize_h, bsize_w;
    int bstride_h, bstride_w;
    int boffset_h, boffset_w;
    int bcount_h, bcount_w;
} sbnet_geom;

/*
 * Compute-tile choices the kernels make from the device-side count of active blocks (Sec. 4, "Choosing the
 * optimal block sizes", carried from the block size to the shapes inside a kernel).  Process-wide, host side,
 * read when a call is enqueued; sbnet_set_tuning(NULL) restores the defaults, which are the crossover points
 * measured on MI355X.  Results never depend on them beyond the rounding order of the weight gradient's sum.
 */
typedef struct {
    /* residual unit: cost of an 8 x 8 sub-tile in eighths of a 16 x 16 one; the size whose cost-weighted rounds of
       work over 256 workgroups are fewer is run (8 x 8: four times the items, a shorter latency chain each).
       Default 3; 0 = always 8 x 8; 1000 = always 16 x 16 where the block allows it. */
    int unit_small_item_cost_eighths;
    /* LDS-tiled 3x3 convolution: cost of a 128-pixel work item in eighths of a 256-pixel one; the shape whose
       cost-weighted rounds of work over 256 CUs are fewer is run.  Default 5; 0 = always 128-pixel items;
       1000 = always 256-pixel items. */
    int conv3_small_item_cost_eighths;
    /* weight gradient: splits of the tile list used = min(launch's, n, f * sqrt(n)) for n active tiles, f given
       here for 3x3 and for 1x1 kernels.  Defaults 8 and 16. */
    int wgrad_split_factor_3x3, wgrad_split_factor_1x1;
} sbnet_tuning;
sbnet_status sbnet_set_tuning(const sbnet_tuning *t);      /* host pointer or NULL */
sbnet_status sbnet_get_tuning(sbnet_tuning *t);            /* host pointer */

/* Last error text of the calling thread (host pointer, valid until the next failing call). */
const char *sbnet_last_error(void);

/*
 * Host helper: fill the input-tile geometry g_in, the output-block geometry g_out and the
 * output extent of a kh x kw convolution with strides (sh, sw) and SAME padding (k-1)/2 on
 * an H x W map cut into bo_h x bo_w output blocks (Sec. 3.1; output extent per Sec. 3.2
 * read as floor((H + 2p - k)/s) + 1).  All pointers are host pointers.
 */
sbnet_status sbnet_geometry(int H, int W, int kh, int kw, int sh, int sw, int bo_h, int bo_w,
                            sbnet_geom *g_in, sbnet_geom *g_out, int *H_out, int *W_out);

/*
 * Geometry of the same block windows on a mask that is given `factor` times coarser and meant to be upsampled by
 * pixel repetition (a mask predicted at lower resolution: Sec. 3.1 reduces "the mask" whatever made it; the
 * benchmark configuration with a 1/8-resolution logit map is the case in point).  Window b of `g` covers the coarse
 * cells its pixels fall into, so
 *     sbnet_reduce_mask(coarse_map, ..., coarse, SBNET_POOL_MAX, t, ...)
 * lists exactly the blocks that thresholding the coarse map at t, upsampling it and reducing the result with `g`
 * (either pooling, threshold 0) lists, for t >= 0 (cells outside the map count as 0 in both), without the
 * upsampled mask ever existing.  Host arithmetic only.  g->bstride_* must be multiples of factor (SBNET_EINVAL).
 */
sbnet_status sbnet_coarse_geometry(const sbnet_geom *g, int factor, sbnet_geom *coarse);

/* Bytes of device scratch sbnet_reduce_mask needs for N samples and geometry g (host call). */
size_t sbnet_workspace_bytes(int N, const sbnet_geom *g);

/*
 * Reduce mask to indices (Sec. 3.1; Sec. 3.4 "fused downsample and indexing").
 * mask: [N][H][W], SBNET_U8 or SBNET_F32.  For every block window of g (pixels outside the
 * image count as 0) the mask is max- or average-pooled (average divides by the full window
 * area) and the block is active when pooled > threshold (strict).  Writes the active
 * (n, by, bx) triples in lexicographic order to indices[0 .. min(count, cap)) and the true
 * number of active blocks to *count (count is overwritten, not accumulated).
 * workspace: device scratch of at least sbnet_workspace_bytes(N, g); contents are don't-care
 * on entry and exit.
 */
sbnet_status sbnet_reduce_mask(const void *mask, sbnet_dtype mask_dtype, int N, int H, int W,
                               const sbnet_geom *g, sbnet_pool pool, float threshold,
                               int32_t *indices, int32_t *count, int cap, void *workspace,
                               size_t workspace_bytes, void *stream);

/*
 * sbnet_reduce_mask for callers that cannot allocate or hand over device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results
 * and kernels as sbnet_reduce_mask, minus the workspace: the row counts and block flags go to a
 * buffer of SBNET_REDUCE_MASK_STATIC_MAX_BYTES that is part of the library's device image (every
 * GPU the library runs on holds its own copy until the process ends).  The call allocates and
 * frees nothing.  Problems whose sbnet_workspace_bytes(N, g) exceeds the buffer are rejected
 * with SBNET_EUNSUPPORTED before anything is enqueued (1 MiB holds e.g. 8 samples of 800 x 704
 * with 8 x 8 blocks fourteen times over).  Nothing in the buffer has to start at zero: every byte
 * the kernels read is written earlier in the same call.  All calls on one GPU share the one
 * buffer, so two calls whose kernels may overlap (different streams, no dependency) race;
 * calls on one stream, or ordered by events, are safe.
 */
#define SBNET_REDUCE_MASK_STATIC_MAX_BYTES ((size_t)1 << 20)
sbnet_status sbnet_reduce_mask_static(const void *mask, sbnet_dtype mask_dtype, int N, int H, int W,
                                      const sbnet_geom *g, sbnet_pool pool, float threshold,
                                      int32_t *indices, int32_t *count, int cap, void *stream);

/*
 * Synchronising helper: copies *count to the host after waiting for `stream`.  Returns
 * SBNET_ECAP (and still stores the true count) when it exceeds cap.
 */
sbnet_status sbnet_read_count(const int32_t *count, int cap, int *host_count, void *stream);

/*
 * Gather (Sec. 3.2 "Gather kernel"): tiles[b][i][j][c] = x[n_b][y0_b + i][x0_b + j][c], zero
 * where the position is outside the H x W image, for b < min(*count, cap).
 * x: [N][H][W][C]; tiles: [cap][g->bsize_h][g->bsize_w][C]; same dtype (F32, BF16 or F16).
 * Rows of tiles beyond the active count are not written.  The copy is bit-exact.
 */
sbnet_status sbnet_sparse_gather(const void *x, sbnet_dtype dtype, int N, int H, int W, int C,
                                 const int32_t *indices, const int32_t *count, int cap,
                                 const sbnet_geom *g, void *tiles, void *stream);

/*
 * Scatter / scatter-add (Sec. 3.2 "Scatter kernel"; Sec. 3.4 "fused scatter-add"):
 * y[n_b][y0_b + i][x0_b + j][c] = (add ? y[...] : 0) + tiles[b][i][j][c] for positions inside
 * the image; nothing else in y is read or written (y is not cleared).  g must describe
 * non-overlapping blocks (bstride >= bsize), otherwise SBNET_EINVAL.  The sum is formed in
 * fp32 and rounded to the storage type (round to nearest even).
 */
sbnet_status sbnet_sparse_scatter(const void *tiles, sbnet_dtype dtype, const int32_t *indices,
                                  const int32_t *count, int cap, const sbnet_geom *g, void *y,
                                  int N, int H, int W, int C, int add, void *stream);

/*
 * Gather and scatter with the transpose fused in (Sec. 3.4 "Fused transpose+gather and
 * transpose+scatter kernels"): the feature map is NHWC as above, the tile stack channel-major,
 * tiles_chw: [cap][C][g->bsize_h][g->bsize_w], for a consumer that wants that layout.
 *   gather_chw:  tiles_chw[b][c][i][j] = x[n_b][y0_b + i][x0_b + j][c], zero outside the image;
 *   scatter_chw: y[n_b][y0_b + i][x0_b + j][c] = (add ? y[...] : 0) + tiles_chw[b][c][i][j] inside
 *                the image, nothing else in y touched; non-overlapping blocks as for
 *                sbnet_sparse_scatter; the sum is formed in fp32 and rounded to nearest even.
 * Bit-exact copies otherwise.  Same dtype on both sides (F32, BF16 or F16); C * element size
 * must be a multiple of 16 bytes and a tile at most 1280 pixels, else SBNET_EUNSUPPORTED.
 */
sbnet_status sbnet_sparse_gather_chw(const void *x, sbnet_dtype dtype, int N, int H, int W, int C,
                                     const int32_t *indices, const int32_t *count, int cap,
                                     const sbnet_geom *g, void *tiles_chw, void *stream);
sbnet_status sbnet_sparse_scatter_chw(const void *tiles_chw, sbnet_dtype dtype,
                                      const int32_t *indices, const int32_t *count, int cap,
                                      const sbnet_geom *g, void *y, int N, int H, int W, int C,
                                      int add, void *stream);

/*
 * Gradient of the gather (end of Sec. 3.3, "End-to-end training of SBNet": the gradient of the
 * overlapping gather is a scatter that adds the tile gradients, also where neighbouring tiles
 * share their halo; the gradient of the scatter is sbnet_sparse_gather itself):
 *   dx[n][y][x][c] += sum over active blocks b whose tile covers (y, x) of
 *                     dtiles[b][y - y0_b][x - x0_b][c],      positions outside the image dropped.
 * dtiles: [cap][g->bsize_h][g->bsize_w][C]; dx: [N][H][W][C], accumulated into (clear it first
 * for a fresh gradient); same dtype (F32, BF16 or F16, C * element size a multiple of 4 bytes).
 * The contributions of a pixel (at most (R+1)^2, R = ceil((bsize - bstride) / bstride) <= 3) are
 * added in ascending (by, bx) order, then dx, in fp32, and rounded once: no atomics, the result
 * does not depend on scheduling.  indices must hold distinct blocks of the g grid (as
 * sbnet_reduce_mask writes them).  workspace: device, sbnet_gather_backward_workspace_bytes(N, g)
 * bytes, 4-byte aligned, overwritten.
 */
size_t sbnet_gather_backward_workspace_bytes(int N, const sbnet_geom *g);
sbnet_status sbnet_sparse_gather_backward(const void *dtiles, sbnet_dtype dtype,
                                          const int32_t *indices, const int32_t *count, int cap,
                                          const sbnet_geom *g, void *dx, int N, int H, int W,
                                          int C, void *workspace, size_t workspace_bytes,
                                          void *stream);

/*
 * Batch-norm statistics over the active blocks only (Sec. 3.3: normalising across the non-sparse
 * elements keeps invalid data out of the statistics): for every channel c,
 *   mean[c] = average, var[c] = biased variance of x[n][y][x][c]
 * over the pixels of the blocks b < min(*count, cap) that lie inside the image (every pixel once:
 * g must describe non-overlapping blocks, else SBNET_EINVAL).  With no such pixel both are 0.
 * x: [N][H][W][C] in `dtype` (F32, BF16 or F16; C * element size a multiple of 16 bytes);
 * mean, var: device float32 [C].  Sums are formed in fp32 in a fixed order (per block, relative to
 * the block's first pixel; blocks merged in a fixed tree): no atomics, the result does not depend on
 * scheduling.  workspace: device, sbnet_bn_stats_workspace_bytes(cap, C) bytes, 4-byte aligned,
 * overwritten.
 */
size_t sbnet_bn_stats_workspace_bytes(int cap, int C);
sbnet_status sbnet_sparse_bn_stats(const void *x, sbnet_dtype dtype, int N, int H, int W, int C,
                                   const int32_t *indices, const int32_t *count, int cap,
                                   const sbnet_geom *g, float *mean, float *var, void *workspace,
                                   size_t workspace_bytes, void *stream);

/*
 * Batch normalisation over the active blocks (Sec. 3.3), forward: for the pixels of the blocks
 * b < min(*count, cap) that lie inside the image,
 *   y = act(gamma[c] * (x - mean[c]) / sqrt(var[c] + eps) + beta[c]),   act = ReLU if relu != 0;
 * every other pixel of y is left as it is.  x, y: [N][H][W][C] in `dtype` (C * element size a
 * multiple of 16 bytes), 16-byte aligned, y may be x; mean, var (e.g. from sbnet_sparse_bn_stats),
 * gamma, beta: device float32 [C], gamma / beta may be NULL (1 / 0).  g: non-overlapping blocks.
 * fp32 arithmetic, one rounding to `dtype`.
 */
sbnet_status sbnet_sparse_bn_apply(const void *x, sbnet_dtype dtype, int N, int H, int W, int C,
                                   const int32_t *indices, const int32_t *count, int cap,
                                   const sbnet_geom *g, const float *mean, const float *var,
                                   const float *gamma, const float *beta, float eps, int relu,
                                   void *y, void *stream);

/*
 * Backward of the call above in training mode, i.e. when mean and var are the statistics of the
 * same active pixels of x (count n).  With xhat = (x - mean) / sqrt(var + eps) and
 * g = dy (relu == 0) or dy where gamma * xhat + beta > 0 and 0 elsewhere (relu != 0):
 *   dbeta[c] = sum g,  dgamma[c] = sum g * xhat   over the active pixels,
 *   dx = gamma / sqrt(var + eps) * (g - dbeta / n - xhat * dgamma / n)   on the active pixels;
 * other pixels of dx are left as they are; dx may be dy.  dgamma, dbeta: device float32 [C],
 * written also when gamma / beta are NULL.  Sums in fp32 in a fixed order (per block, then a fixed
 * tree over the blocks): no atomics.  workspace: device, 4-byte aligned,
 * sbnet_bn_backward_workspace_bytes(cap, C) bytes, overwritten.
 */
size_t sbnet_bn_backward_workspace_bytes(int cap, int C);
sbnet_status sbnet_sparse_bn_backward(const void *x, const void *dy, sbnet_dtype dtype, int N, int H,
                                      int W, int C, const int32_t *indices, const int32_t *count,
                                      int cap, const sbnet_geom *g, const float *mean,
                                      const float *var, const float *gamma, const float *beta,
                                      float eps, int relu, void *dx, float *dgamma, float *dbeta,
                                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * Re-pack convolution weights once for the kernels below.  w_hwio: device, [kh][kw][Cin][Cout]
 * in `dtype` (the filter bank as a (kh*kw*Cin) x Cout matrix, Sec. 2).  With w_packed == NULL
 * only *bytes (host) is set to the size the packed copy needs.  The packed layout is private
 * to the library and depends only on (dtype, kh, kw, Cin, Cout).
 */
sbnet_status sbnet_pack_weights(const void *w_hwio, sbnet_dtype dtype, int kh, int kw, int Cin,
                                int Cout, void *w_packed, size_t *bytes, void *stream);

/*
 * Regular unpadded convolution on the tile stack (Sec. 3.2): cross-correlation,
 * out[b][i][j][o] = act(bias[o] + sum_{r,t,c} in[b][i*sh + r][j*sw + t][c] * w[r][t][c][o]),
 * output extent floor((th - kh)/sh) + 1 by floor((tw - kw)/sw) + 1, act = ReLU when relu != 0.
 * tiles_in: [cap][th][tw][Cin]; tiles_out: [cap][th'][tw'][Cout]; both `dtype`.
 * bias: device float32 [Cout] or NULL.  Products are accumulated in fp32.
 */
sbnet_status sbnet_conv_on_tiles(const void *tiles_in, sbnet_dtype dtype, const int32_t *count,
                                 int cap, int th, int tw, int Cin, const void *w_packed,
                                 const float *bias, int kh, int kw, int sh, int sw, int Cout,
                                 int relu, void *tiles_out, void *stream);

/*
 * Fused gather -> convolution -> scatter(-add) (Fig. 1 in one kernel): same result as
 * sbnet_sparse_gather with g_in, sbnet_conv_on_tiles, sbnet_sparse_scatter with g_out, except
 * that the convolution result is not rounded to `dtype` before the add; the intermediate tile
 * stacks never exist.  x: [N][H][W][Cin]; y: [N][H_out][W_out][Cout].
 * g_in/g_out as produced by sbnet_geometry for this convolution.  y must not overlap x (not even in part).
 */
sbnet_status sbnet_sparse_conv(const void *x, sbnet_dtype dtype, int N, int H, int W, int Cin,
                               const int32_t *indices, const int32_t *count, int cap,
                               const sbnet_geom *g_in, const sbnet_geom *g_out,
                               const void *w_packed, const float *bias, int kh, int kw, int sh,
                               int sw, int Cout, int relu, void *y, int H_out, int W_out,
                               int add, void *stream);

/*
 * The pooling half of reduce_mask on its own (Sec. 3.1; Sec. 3.4 "fused downsample and indexing" stops
 * one step earlier): flags[blk] = 1 where block blk = (n * bcount_h + by) * bcount_w + bx is active
 * (same pooling and threshold rule as sbnet_reduce_mask), else 0, for every block of the grid.
 * flags: device, sbnet_block_flags_bytes(N, g) bytes (one per block, rounded up to 16; the bytes behind
 * the last block are written as 0), 16-byte aligned.
 * Grids of more than 65 536 blocks return SBNET_EUNSUPPORTED (use sbnet_reduce_mask).
 */
size_t sbnet_block_flags_bytes(int N, const sbnet_geom *g);
sbnet_status sbnet_block_flags(const void *mask, sbnet_dtype mask_dtype, int N, int H, int W,
                               const sbnet_geom *g, sbnet_pool pool, float threshold, uint8_t *flags,
                               size_t flags_bytes, void *stream);

/*
 * sbnet_sparse_conv fed by the block flags instead of the index list (Fig. 1 with the second half of
 * Sec. 3.1 moved into the consumer): the same y as sbnet_sparse_conv on the list those flags compact to,
 * and that list and its count are written to indices / count for later calls.  Where the convolution
 * kernel can take flags (3x3, stride 1, 16 x 16 output blocks, 32 or 64 input channels, bf16 / f16) every
 * workgroup compacts them in its prologue while its weights arrive, which saves reduce_mask's second
 * launch; every other shape compacts the flags in a launch of its own and runs sbnet_sparse_conv.
 * The block grid of g_in and g_out is the one the flags were made for; at most 65 536 blocks.  flags is
 * what sbnet_block_flags writes: every byte 0 or 1, sbnet_block_flags_bytes(N, g_in) of them, zero behind
 * the last block.
 */
sbnet_status sbnet_sparse_conv_from_flags(const uint8_t *flags, const void *x, sbnet_dtype dtype, int N,
                                          int H, int W, int Cin, int32_t *indices, int32_t *count, int cap,
                                          const sbnet_geom *g_in, const sbnet_geom *g_out,
                                          const void *w_packed, const float *bias, int kh, int kw, int sh,
                                          int sw, int Cout, int relu, void *y, int H_out, int W_out, int add,
                                          void *stream);

/*
 * Mask in, convolved active blocks out, in one call (Fig. 1 end to end): sbnet_block_flags into the
 * workspace followed by sbnet_sparse_conv_from_flags; grids beyond 65 536 blocks run sbnet_reduce_mask and
 * sbnet_sparse_conv.  Same results as those calls, in y and in indices / count.
 * mask: [N][mask_H][mask_W] (u8 or f32), pooled over the windows of g_mask, whose block grid must be that
 * of g_in and g_out (for a stride-1 convolution the mask has the input's extent and g_mask is g_in or the
 * output-block geometry).  workspace: at least sbnet_workspace_bytes(N, g_mask), 16-byte aligned, contents
 * don't-care.  All other arguments as in the calls it stands for.
 */
sbnet_status sbnet_sparse_conv_from_mask(const void *mask, sbnet_dtype mask_dtype, int mask_H, int mask_W,
                                         const sbnet_geom *g_mask, sbnet_pool pool, float threshold,
                                         const void *x, sbnet_dtype dtype, int N, int H, int W, int Cin,
                                         int32_t *indices, int32_t *count, int cap,
                                         const sbnet_geom *g_in, const sbnet_geom *g_out,
                                         const void *w_packed, const float *bias, int kh, int kw, int sh,
                                         int sw, int Cout, int relu, void *y, int H_out, int W_out, int add,
                                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * Data gradient of sbnet_conv_on_tiles (training support for the tile convolution of Sec. 3.2;
 * the paper's own evaluation is inference only).  For y = valid convolution of x with W at stride
 * (sh, sw), no bias and no activation, and a given dL/dy this writes
 *   din[b][y][x][c] = sum over (r, t, o) with (y - r) % sh == 0, (x - t) % sw == 0 and the quotients
 *                     inside the output tile of  W[r][t][c][o] * dout[b][(y - r)/sh][(x - t)/sw][o],
 * rounded once to `dtype` (fp32 accumulation; BF16/F16 contractions on the matrix cores).  A ReLU
 * in the forward call is the caller's to undo (mask dout by y > 0 first); the bias gradient is a
 * plain sum of dout.
 * dout_tiles: [cap][oh][ow][Cout] with oh = (th - kh)/sh + 1, ow likewise; din_tiles:
 * [cap][th][tw][Cin], every element of the tiles b < min(*count, cap) written (input rows a strided
 * window never reaches get 0).  w_packed_t: from sbnet_pack_weights_transposed, called with the
 * forward convolution's w_hwio, kh, kw, Cin, Cout.  workspace: device, 16-byte aligned,
 * sbnet_conv_backward_data_workspace_bytes(...) bytes (at strides above 1 the output gradient spread
 * by the stride and framed by kh-1 / kw-1 zeros, [cap][th+kh-1][tw+kw-1][Cout]; at stride 1 only
 * one index triple per tile); overwritten.  All pointers device
 * and 16-byte aligned.  Feeding din_tiles to sbnet_sparse_gather_backward gives dL/dx of the whole
 * sparse convolution; dout_tiles come from sbnet_sparse_gather of dL/dy with the output geometry.
 */
sbnet_status sbnet_pack_weights_transposed(const void *w_hwio, sbnet_dtype dtype, int kh, int kw,
                                           int Cin, int Cout, void *w_packed, size_t *bytes,
                                           void *stream);
size_t sbnet_conv_backward_data_workspace_bytes(sbnet_dtype dtype, int cap, int th, int tw, int kh,
                                                int kw, int sh, int sw, int Cout);
sbnet_status sbnet_conv_on_tiles_backward_data(const void *dout_tiles, sbnet_dtype dtype,
                                               const int32_t *count, int cap, int th, int tw,
                                               int Cin, const void *w_packed_t, int kh, int kw,
                                               int sh, int sw, int Cout, void *din_tiles,
                                               void *workspace, size_t workspace_bytes,
                                               void *stream);

/*
 * Weight gradient of sbnet_conv_on_tiles (training support, as above): with the forward input
 * tiles x and dL/dy on tiles,
 *   dw[r][t][c][o] = sum over b < min(*count, cap) and output pixels (i, j) of
 *                    x[b][r + sh*i][t + sw*j][c] * dout[b][i][j][o],
 * written (not added) to dw: device float32 [kh][kw][Cin][Cout]; all zeros when no tile is
 * active.  tiles_in: [cap][th][tw][Cin], dout_tiles: [cap][oh][ow][Cout] in `dtype` (F32, BF16 or
 * F16), 16-byte aligned.  Products of BF16/F16 inputs are exact and summed in fp32; the tiles are
 * split over workgroups whose partial sums are added in a fixed order (no atomics: the same
 * inputs give the same bits).  3x3 and 1x1 kernels at stride 1 or 2 with channel counts that are
 * multiples of 8 (output tiles up to 32 columns; any tile for 1x1 at stride 1) run on the matrix
 * cores, everything else in a plain kernel (correct, slow).  workspace: device, 16-byte aligned,
 * sbnet_conv_backward_weights_workspace_bytes(...) bytes (the partial sums); overwritten.
 */
size_t sbnet_conv_backward_weights_workspace_bytes(sbnet_dtype dtype, int cap, int th, int tw,
                                                   int Cin, int kh, int kw, int sh, int sw,
                                                   int Cout);
sbnet_status sbnet_conv_on_tiles_backward_weights(const void *tiles_in, const void *dout_tiles,
                                                  sbnet_dtype dtype, const int32_t *count, int cap,
                                                  int th, int tw, int Cin, int kh, int kw, int sh,
                                                  int sw, int Cout, float *dw, void *workspace,
                                                  size_t workspace_bytes, void *stream);

/*
 * The two element-wise pieces a backward pass through a chain of tile convolutions needs besides
 * the convolutions' own gradients (the residual unit of Sec. 3.3 composed from single calls).
 *
 * sbnet_relu_backward_on_tiles: dout = dy where the forward activation y is > 0, else 0, on the tiles
 * b < min(*count, cap) of stacks with tile_elems elements per tile (a whole number of 4-byte words);
 * later tiles are not touched; dout may be dy.  Device pointers, 16-byte aligned.
 *
 * sbnet_bias_backward_on_tiles: db[c] = sum over those tiles and their `pixels` pixels of dy[b][pixel][c]
 * (the gradient of the bias a convolution adds), device float32 [C], zeros when no tile is active.
 * fp32 sums in a fixed order, no atomics.  C * element size a multiple of 4 bytes and at most 1 KiB
 * (4 KiB where it is a multiple of 16 bytes and dy_tiles is 16-byte aligned).
 * workspace: device, 4-byte aligned, sbnet_bias_backward_workspace_bytes(cap, C) bytes, overwritten.
 *
 * sbnet_relu_bias_backward_on_tiles: both in one pass over the gradient that enters a convolution
 * through its ReLU: dout = dy where y > 0, else 0, and db[c] = the sum of dout over the active tiles
 * and their pixels; same results, bit for bit, as the two calls above in that order.  Tiles of
 * `pixels` pixels with C channels; dout may be dy; limits and workspace as for
 * sbnet_bias_backward_on_tiles (16-byte accesses need all three stacks 16-byte aligned).
 */
sbnet_status sbnet_relu_backward_on_tiles(const void *y_tiles, const void *dy_tiles, sbnet_dtype dtype,
                                          const int32_t *count, int cap, size_t tile_elems,
                                          void *dout_tiles, void *stream);
size_t sbnet_bias_backward_workspace_bytes(int cap, int C);
sbnet_status sbnet_bias_backward_on_tiles(const void *dy_tiles, sbnet_dtype dtype, const int32_t *count,
                                          int cap, int pixels, int C, float *db, void *workspace,
                                          size_t workspace_bytes, void *stream);
sbnet_status sbnet_relu_bias_backward_on_tiles(const void *y_tiles, const void *dy_tiles,
                                               sbnet_dtype dtype, const int32_t *count, int cap,
                                               int pixels, int C, void *dout_tiles, float *db,
                                               void *workspace, size_t workspace_bytes,
                                               void *stream);

/*
 * FP8 variant of the tile convolution (the paper fixes no precision for the convolution between
 * gather and scatter, Sec. 3.2).  Storage is FP8 E4M3 in the OCP "e4m3fn" encoding (sign, 4 exponent
 * bits with bias 7, 3 mantissa bits; no infinities; 0x7f / 0xff are NaN; largest finite value 448).
 *
 * sbnet_quantize_f8: out[i] = e4m3(clamp(x[i] * scale, -448, 448)), round to nearest even (the product
 * in fp32), for `elems` elements of any F32 / BF16 / F16 device buffer; out: device bytes.
 *
 * sbnet_pack_weights_f8: w_hwio_f8 [kh][kw][Cin][Cout] bytes -> the private operand order; size query
 * as sbnet_pack_weights.
 *
 * sbnet_conv_on_tiles_f8: tiles_out[b] = act(out_scale * (valid convolution of tiles_in[b] with w) +
 * bias) for b < min(*count, cap): products of the decoded FP8 values are exact, summed in fp32 on the
 * matrix cores; out_scale (finite) undoes the scales inputs and weights were quantised with; the
 * result is rounded once to BF16.  tiles_in: [cap][th][tw][Cin] bytes; tiles_out:
 * [cap][oh][ow][Cout] BF16; bias: float32 [Cout] or NULL.  Cin % 16 == 0, Cout % 8 == 0, else
 * SBNET_EUNSUPPORTED.  Device pointers, 16-byte aligned.
 */
sbnet_status sbnet_quantize_f8(const void *x, sbnet_dtype dtype, size_t elems, float scale, void *out,
                               void *stream);
sbnet_status sbnet_pack_weights_f8(const void *w_hwio_f8, int kh, int kw, int Cin, int Cout,
                                   void *w_packed, size_t *bytes, void *stream);
sbnet_status sbnet_conv_on_tiles_f8(const void *tiles_in_f8, const int32_t *count, int cap, int th,
                                    int tw, int Cin, const void *w_packed_f8, const float *bias,
                                    int kh, int kw, int sh, int sw, int Cout, int relu,
                                    float out_scale, void *tiles_out_bf16, void *stream);

/*
 * Backward pass of the residual branch of a bottleneck unit on tiles (Sec. 3.3; the forward branch is
 * sbnet_bottleneck_on_tiles), composed from the calls above; nothing but they runs.  The caller keeps
 * the forward activations t1 = ReLU(W1 x + b1) with the positions outside the image set to zero
 * ([cap][th][tw][Cm]) and t2 = ReLU(W2 * t1 + b2) ([cap][th-2][tw-2][Cm]) - a training forward pass
 * runs the three convolutions as single calls, the fused kernel does not keep them - and passes
 * dt3 = dL/dt3 ([cap][th-2][tw-2][C]).  Written: dtiles_in = dL/dx on the input tiles ([cap][th][tw][C],
 * `dtype`), and in float32 dw1 [1][1][C][Cm], db1 [Cm], dw2 [3][3][Cm][Cm], db2 [Cm], dw3 [1][1][Cm][C],
 * db3 [C], each summed over the tiles b < min(*count, cap).  w1_t, w2_t, w3_t: the three forward weight
 * arrays packed by sbnet_pack_weights_transposed.  workspace: device, 256-byte aligned,
 * sbnet_bottleneck_backward_workspace_bytes(...) bytes, overwritten (it holds dL/dt2, dL/dt1 and the
 * scratch of the single calls).  The unit's identity path adds dL/dy to dL/dx outside this call.
 */
/*
 * The forward pass that keeps what the call below needs: the residual branch of sbnet_bottleneck_on_tiles
 * as its three convolutions in single calls, writing t1 (with the positions outside the H x W image set
 * to zero, [cap][th][tw][Cm]), t2 ([cap][th-2][tw-2][Cm]) and t3 ([cap][th-2][tw-2][C]).  Weights from
 * sbnet_pack_weights, biases float32 or NULL; any element type and channel counts the tile convolution
 * takes.  th, tw = g_in->bsize.  The results equal the fused kernel's up to its rounding of t1 and t2.
 */
sbnet_status sbnet_bottleneck_forward_keep_on_tiles(const void *tiles_in, sbnet_dtype dtype, int H, int W,
                                                    int C, int Cm, const int32_t *indices,
                                                    const int32_t *count, int cap,
                                                    const sbnet_geom *g_in, const void *w1,
                                                    const float *b1, const void *w2, const float *b2,
                                                    const void *w3, const float *b3, void *t1, void *t2,
                                                    void *t3, void *stream);
size_t sbnet_bottleneck_backward_workspace_bytes(sbnet_dtype dtype, int cap, int th, int tw, int C,
                                                 int Cm);
sbnet_status sbnet_bottleneck_backward_on_tiles(const void *tiles_in, const void *t1, const void *t2,
                                                const void *dt3, sbnet_dtype dtype,
                                                const int32_t *count, int cap, int th, int tw, int C,
                                                int Cm, const void *w1_t, const void *w2_t,
                                                const void *w3_t, void *dtiles_in, float *dw1,
                                                float *db1, float *dw2, float *db2, float *dw3,
                                                float *db3, void *workspace, size_t workspace_bytes,
                                                void *stream);

/*
 * Sparse residual unit of any width, stride and shortcut (Sec. 3.3; the downsampling units of the backbone
 * of Sec. 4; strided tile geometry of Sec. 3.1 / Fig. 3).  On the active output blocks
 *     y = shortcut(x) + W3 ReLU(W2 *_s t1 + b2) + b3,   t1 = ReLU(W1 x + b1), zero outside the image,
 * W1: 1x1 Cin -> Cm, W2: 3x3 with `stride` and padding 1, Cm -> Cm, W3: 1x1 Cm -> Cout (all from
 * sbnet_pack_weights; biases device float32, required).  shortcut: w_shortcut / b_shortcut = a 1x1
 * convolution Cin -> Cout with the same stride (packed the same way), or both NULL = the identity (needs
 * stride 1 and Cin == Cout).  Pixels of y outside the active blocks are neither read nor written.
 * x: [N][H][W][Cin]; y: [N][H_out][W_out][Cout]; g_in / g_out from sbnet_geometry(H, W, 3, 3, stride, stride, ...).
 * y may be x only with the identity shortcut (the in-place scatter-add of Sec. 3.4).
 * One launch, no workspace (it may be NULL), bf16 / f16, block sides multiples of 8, y != x:
 *   - stride 1 with the identity: the shapes of sbnet_sparse_bottleneck (Cin in {64, 96, 128, 192, 256} with
 *     Cm <= 64, Cin = 384 with Cm in 72 .. 96);
 *   - stride 2 with a projected shortcut: Cin -> Cout in {64 -> 96, 96 -> 192, 192 -> 256, 64 -> 128, 128 -> 256}
 *     with Cm <= 64, and 256 -> 384 with Cm in 72 .. 96 (the four downsampling units of the backbone of Sec. 4).
 *   There x + branch (or shortcut + branch) is formed in fp32 and rounded once; t1 and t2 are rounded to `dtype`.
 * Every other shape runs as gather, the three convolutions on tile stacks, the shortcut and one scatter-add, on
 * tile stacks in `workspace` (sbnet_sparse_unit_workspace_bytes, 256-byte aligned, contents don't-care): t1, t2
 * and t3 are rounded to `dtype` between the steps, the shortcut is rounded before the branch is added.
 */
size_t sbnet_sparse_unit_workspace_bytes(sbnet_dtype dtype, int cap, const sbnet_geom *g_in,
                                         const sbnet_geom *g_out, int Cin, int Cm, int Cout);
sbnet_status sbnet_sparse_unit(const void *x, sbnet_dtype dtype, int N, int H, int W, int Cin, int Cm,
                               int Cout, int stride, const int32_t *indices, const int32_t *count, int cap,
                               const sbnet_geom *g_in, const sbnet_geom *g_out, const void *w1,
                               const float *b1, const void *w2, const float *b2, const void *w3,
                               const float *b3, const void *w_shortcut, const float *b_shortcut, void *y,
                               int H_out, int W_out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Set every tile position that lies outside the H x W image to zero, in place.  Needed when a
 * residual unit is composed from single sbnet_conv_on_tiles calls: after the first convolution
 * the halo positions beyond the image border hold act(bias), but the next convolution's zero
 * padding applies to that activation (Sec. 3.3 leaves the image border implicit).
 * tiles: [cap][g->bsize_h][g->bsize_w][C].
 */
sbnet_status sbnet_zero_outside(void *tiles, sbnet_dtype dtype, int H, int W, int C,
                                const int32_t *indices, const int32_t *count, int cap,
                                const sbnet_geom *g, void *stream);

/*
 * Residual branch of a sparse bottleneck unit on gathered tiles (Sec. 3.3, Fig. 4; batch norm
 * folded into weights and biases): t1 = ReLU(W1 x + b1) (1x1, C -> Cm) on the whole input tile,
 * set to zero at tile positions outside the H x W image (the 3x3 of the dense network pads its
 * own input with zeros); t2 = ReLU(W2 * t1 + b2) (3x3 unpadded, Cm -> Cm); t3 = W3 t2 + b3
 * (1x1, Cm -> C).  tiles_in: [cap][g_in->bsize_h][g_in->bsize_w][C] as written by
 * sbnet_sparse_gather; tiles_out: [cap][g_out->bsize_h][g_out->bsize_w][C] receives t3, ready for
 * sbnet_sparse_scatter with add = 1.  indices and the geometries locate each tile in the image
 * for the border rule.  w1, w2, w3 come from sbnet_pack_weights (shapes [1][1][C][Cm],
 * [3][3][Cm][Cm], [1][1][Cm][C]); b1, b2, b3 are device float32 and required.  t1 and t2 are
 * rounded to `dtype` between the layers; sums are fp32.
 * Supported: bf16 / f16, C in {64, 96, 128, 192, 256}, Cm a multiple of 8 up to 64 (the unit widths of
 * the detector backbone of Sec. 4 up to its third stage: 96/24, 192/48, 256/64), block sides multiples
 * of 8, input tile = block + one-pixel halo, one tile below 2^30 elements; the fused call
 * sbnet_sparse_bottleneck also takes the fourth stage's C = 384 with Cm a multiple of 8 in 72 .. 96; anything
 * else returns SBNET_EUNSUPPORTED (sbnet_sparse_unit takes every width, strides and projected shortcuts).
 */
sbnet_status sbnet_bottleneck_on_tiles(const void *tiles_in, sbnet_dtype dtype, int H, int W, int C,
                                       int Cm, const int32_t *indices, const int32_t *count, int cap,
                                       const sbnet_geom *g_in, const sbnet_geom *g_out,
                                       const void *w1, const float *b1, const void *w2,
                                       const float *b2, const void *w3, const float *b3,
                                       void *tiles_out, void *stream);

/*
 * Whole sparse residual unit in one kernel: one gather, three convolutions, one scatter-add
 * (Sec. 3.3, Sec. 3.4): y = x + t3 on the pixels of active blocks, with t3 as defined above.
 * x, y: [N][H][W][C].  Pixels of inactive blocks of y are neither read nor written.
 * The paper adds the result onto the input tensor in place; a single fused kernel cannot,
 * because a block's halo overlaps its neighbours' output pixels.  y must therefore be a second
 * buffer (SBNET_EINVAL if y == x).  For a stack of units sharing one index list, initialise
 * both buffers with the input once and alternate them: inactive pixels never change, and every
 * active pixel of the buffer being read was written by the previous unit.
 * x + t3 is formed in fp32 and rounded to `dtype` once (the route over sbnet_bottleneck_on_tiles and
 * sbnet_sparse_scatter rounds t3 for its tile stack and the sum again: at most half a unit in the last place of
 * t3 plus one of the sum apart).
 * Support matrix of sbnet_bottleneck_on_tiles plus C = 384 with Cm in 72 .. 96; one sample (H * W * C) below
 * 2^30 elements.
 */
sbnet_status sbnet_sparse_bottleneck(const void *x, sbnet_dtype dtype, int N, int H, int W, int C,
                                     int Cm, const int32_t *indices, const int32_t *count, int cap,
                                     const sbnet_geom *g_in, const sbnet_geom *g_out,
                                     const void *w1, const float *b1, const void *w2,
                                     const float *b2, const void *w3, const float *b3, void *y,
                                     void *stream);

/*
 * The same unit in pre-activation form: a per-channel affine map and ReLU (a batch norm folded to
 * scale and shift, then ReLU) sit in front of the first convolution, the residual stays x:
 *   y = x + W3 * ReLU(W2 (*) ReLU(W1 * ReLU(pre_scale . x + pre_shift) + b1) + b2) + b3
 * on the active blocks (Sec. 3.3 names the unit's layers - three convolutions, batch
 * normalisation, ReLU - without fixing their order; this is the order of pre-activation
 * residual networks).  pre_scale, pre_shift: device float32 [C].  Everything else as for
 * sbnet_bottleneck_on_tiles / sbnet_sparse_bottleneck, including the support matrix (without C = 384); the
 * fused form rounds t3 before the add, as the route over the tile stack does (same bits).
 */
sbnet_status sbnet_bottleneck_on_tiles_preact(const void *tiles_in, sbnet_dtype dtype, int H, int W,
                                              int C, int Cm, const int32_t *indices,
                                              const int32_t *count, int cap, const sbnet_geom *g_in,
                                              const sbnet_geom *g_out, const float *pre_scale,
                                              const float *pre_shift, const void *w1, const float *b1,
                                              const void *w2, const float *b2, const void *w3,
                                              const float *b3, void *tiles_out, void *stream);
sbnet_status sbnet_sparse_bottleneck_preact(const void *x, sbnet_dtype dtype, int N, int H, int W,
                                            int C, int Cm, const int32_t *indices,
                                            const int32_t *count, int cap, const sbnet_geom *g_in,
                                            const sbnet_geom *g_out, const float *pre_scale,
                                            const float *pre_shift, const void *w1, const float *b1,
                                            const void *w2, const float *b2, const void *w3,
                                            const float *b3, void *y, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SBNET_H */
