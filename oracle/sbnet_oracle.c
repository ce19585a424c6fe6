/*
 * CPU oracle for the tiled sparse convolution of "SBNet: Sparse Blocks Network for
 * Fast Inference" (arXiv 1801.02108).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, single-threaded,
 * double-precision statement of what each step of the method computes, written so it can
 * be checked against the paper by eye.  It shares no code with the GPU library and may be
 * used only by the tests, the smoke check and the benchmark's CPU-baseline leg.
 *
 * All tensors are dense row-major doubles in NHWC order; indices are int32 triples
 * (n, by, bx) of block-grid coordinates.  Nothing here is blocked, fused or reordered.
 *
 * Block geometry (Sec. 3.1, Fig. 3): a block with grid coordinates (by, bx) covers rows
 *   [off_h + by*stride_h, off_h + by*stride_h + size_h)
 * and likewise for columns.  For the input of a k x k, stride-s, SAME-padded convolution
 * with output blocks of bo pixels: size = (bo-1)*s + k, stride = bo*s, off = -(k-1)/2, so
 * neighbouring input tiles overlap by k - s pixels (the quantity Fig. 3 computes as 3-2=1).
 * For the output: size = stride = bo, off = 0 (non-overlapping, Sec. 3.1).
 */
#include <stdint.h>
#include <stddef.h>

typedef struct {
    int size_h, size_w;     /* window / tile extent in pixels                 */
    int stride_h, stride_w; /* distance between origins of neighbouring blocks */
    int off_h, off_w;       /* origin of block (0, 0); may be negative          */
    int count_h, count_w;   /* number of blocks along each axis                 */
} orc_geom;

/*
 * Reduce mask to indices (Sec. 3.1 "Reduce mask to indices"; Sec. 3.4 "Fused downsample
 * and indexing kernel").  For every block window: pool the mask (pool = 0: maximum,
 * pool = 1: average over the full window area, pixels outside the image counting as 0),
 * and keep the block when the pooled value is strictly greater than the threshold.
 * Blocks are visited, and therefore listed, in lexicographic (n, by, bx) order.
 * Returns the number of active blocks; at most `cap` triples are stored.
 */
int orc_reduce_mask(const double *mask, int N, int H, int W, const orc_geom *g, int pool,
                    double threshold, int32_t *indices, int cap)
{
    int count = 0;
    for (int n = 0; n < N; ++n)
        for (int by = 0; by < g->count_h; ++by)
            for (int bx = 0; bx < g->count_w; ++bx) {
                int y0 = g->off_h + by * g->stride_h;
                int x0 = g->off_w + bx * g->stride_w;
                double vmax = 0.0, vsum = 0.0;
                int first = 1;
                for (int i = 0; i < g->size_h; ++i)
                    for (int j = 0; j < g->size_w; ++j) {
                        int y = y0 + i, x = x0 + j;
                        double v = 0.0;
                        if (y >= 0 && y < H && x >= 0 && x < W)
                            v = mask[((size_t)n * H + y) * W + x];
                        vsum += v;
                        if (first || v > vmax) vmax = v;
                        first = 0;
                    }
                double pooled = pool == 0 ? vmax : vsum / ((double)g->size_h * (double)g->size_w);
                if (pooled > threshold) {
                    if (count < cap) {
                        indices[3 * count + 0] = n;
                        indices[3 * count + 1] = by;
                        indices[3 * count + 2] = bx;
                    }
                    ++count;
                }
            }
    return count;
}

/*
 * Gather (Sec. 3.2 "Gather kernel"): slice a size_h x size_w x C window out of the
 * N x H x W x C tensor for every listed block and stack the slices along a new leading
 * axis.  Window positions outside the image read as zero (the SAME padding of the
 * convolution that follows).
 */
void orc_gather(const double *x, int N, int H, int W, int C, const int32_t *indices, int B,
                const orc_geom *g, double *tiles)
{
    (void)N;
    for (int b = 0; b < B; ++b) {
        int n = indices[3 * b], by = indices[3 * b + 1], bx = indices[3 * b + 2];
        int y0 = g->off_h + by * g->stride_h;
        int x0 = g->off_w + bx * g->stride_w;
        for (int i = 0; i < g->size_h; ++i)
            for (int j = 0; j < g->size_w; ++j)
                for (int c = 0; c < C; ++c) {
                    int y = y0 + i, xx = x0 + j;
                    double v = 0.0;
                    if (y >= 0 && y < H && xx >= 0 && xx < W)
                        v = x[(((size_t)n * H + y) * W + xx) * C + c];
                    tiles[(((size_t)b * g->size_h + i) * g->size_w + j) * C + c] = v;
                }
    }
}

/*
 * Scatter and scatter-add (Sec. 3.2 "Scatter kernel"; Sec. 3.4 "Fused scatter-add kernel
 * for residual blocks"): the inverse of gather.  Every tile is written (add = 0) or added
 * (add = 1) to its block of y; positions that fall outside the image are dropped and no
 * other element of y is touched.
 */
void orc_scatter(const double *tiles, const int32_t *indices, int B, const orc_geom *g,
                 double *y, int N, int H, int W, int C, int add)
{
    (void)N;
    for (int b = 0; b < B; ++b) {
        int n = indices[3 * b], by = indices[3 * b + 1], bx = indices[3 * b + 2];
        int y0 = g->off_h + by * g->stride_h;
        int x0 = g->off_w + bx * g->stride_w;
        for (int i = 0; i < g->size_h; ++i)
            for (int j = 0; j < g->size_w; ++j) {
                int yy = y0 + i, xx = x0 + j;
                if (yy < 0 || yy >= H || xx < 0 || xx >= W) continue;
                for (int c = 0; c < C; ++c) {
                    double v = tiles[(((size_t)b * g->size_h + i) * g->size_w + j) * C + c];
                    size_t o = (((size_t)n * H + yy) * W + xx) * C + c;
                    if (add) y[o] += v; else y[o] = v;
                }
            }
    }
}

/*
 * Unpadded ("valid") convolution of a stack of tiles (Sec. 3.2): cross-correlation, no
 * kernel flip, weights in HWIO order w[r][t][c][o].
 *   out[b][i][j][o] = bias[o] + sum_{r,t,c} in[b][i*sh + r][j*sw + t][c] * w[r][t][c][o]
 * with output extent floor((h - kh)/sh) + 1, which for stride 1 is the h - kh + 1 the
 * paper prints.  relu != 0 clamps negatives to zero.  bias may be NULL (zero).
 */
void orc_conv_valid(const double *in, int B, int h, int w_in, int Cin, const double *w,
                    const double *bias, int kh, int kw, int sh, int sw, int Cout, int relu,
                    double *out)
{
    int ho = (h - kh) / sh + 1, wo = (w_in - kw) / sw + 1;
    for (int b = 0; b < B; ++b)
        for (int i = 0; i < ho; ++i)
            for (int j = 0; j < wo; ++j)
                for (int o = 0; o < Cout; ++o) {
                    double acc = bias ? bias[o] : 0.0;
                    for (int r = 0; r < kh; ++r)
                        for (int t = 0; t < kw; ++t)
                            for (int c = 0; c < Cin; ++c)
                                acc += in[(((size_t)b * h + (i * sh + r)) * w_in + (j * sw + t)) * Cin + c] *
                                       w[(((size_t)r * kw + t) * Cin + c) * Cout + o];
                    if (relu && acc < 0.0) acc = 0.0;
                    out[(((size_t)b * ho + i) * wo + j) * Cout + o] = acc;
                }
}

/*
 * Dense zero-padded convolution of the whole feature map: the plain definition the
 * tiled method must reproduce on active blocks (Sec. 3.2, "locally-equivalent to a dense
 * convolution").  Padding ph, pw on every side; output extent floor((H + 2ph - kh)/sh) + 1.
 */
void orc_conv_dense(const double *x, int N, int H, int W, int Cin, const double *w,
                    const double *bias, int kh, int kw, int sh, int sw, int ph, int pw,
                    int Cout, int relu, double *out)
{
    int Ho = (H + 2 * ph - kh) / sh + 1, Wo = (W + 2 * pw - kw) / sw + 1;
    for (int n = 0; n < N; ++n)
        for (int i = 0; i < Ho; ++i)
            for (int j = 0; j < Wo; ++j)
                for (int o = 0; o < Cout; ++o) {
                    double acc = bias ? bias[o] : 0.0;
                    for (int r = 0; r < kh; ++r)
                        for (int t = 0; t < kw; ++t) {
                            int y = i * sh + r - ph, xx = j * sw + t - pw;
                            if (y < 0 || y >= H || xx < 0 || xx >= W) continue;
                            for (int c = 0; c < Cin; ++c)
                                acc += x[(((size_t)n * H + y) * W + xx) * Cin + c] *
                                       w[(((size_t)r * kw + t) * Cin + c) * Cout + o];
                        }
                    if (relu && acc < 0.0) acc = 0.0;
                    out[(((size_t)n * Ho + i) * Wo + j) * Cout + o] = acc;
                }
}

/*
 * Zero every tile position that lies outside the image.  Used between the first and the
 * second convolution of a residual unit run on gathered tiles: in the dense network the
 * 3x3 convolution pads its own input (the activation after the first convolution) with
 * zeros, so positions beyond the image border must be zero there as well, not
 * relu(bias).  The paper does not discuss the image border inside a unit (Sec. 3.3).
 */
void orc_zero_outside(double *tiles, const int32_t *indices, int B, const orc_geom *g, int H,
                      int W, int C)
{
    for (int b = 0; b < B; ++b) {
        int by = indices[3 * b + 1], bx = indices[3 * b + 2];
        int y0 = g->off_h + by * g->stride_h;
        int x0 = g->off_w + bx * g->stride_w;
        for (int i = 0; i < g->size_h; ++i)
            for (int j = 0; j < g->size_w; ++j) {
                int y = y0 + i, xx = x0 + j;
                if (y >= 0 && y < H && xx >= 0 && xx < W) continue;
                for (int c = 0; c < C; ++c)
                    tiles[(((size_t)b * g->size_h + i) * g->size_w + j) * C + c] = 0.0;
            }
    }
}
