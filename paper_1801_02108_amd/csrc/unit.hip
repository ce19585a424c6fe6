// Sparse residual unit of any width, with a strided 3x3 and a projected shortcut (the downsampling units that open
// the stages of the detector backbone, Sec. 4 "Architecture" of arXiv 1801.02108; a unit shares one gather and one
// scatter, Sec. 3.3; the strided tile is that of Sec. 3.1 / Fig. 3: input side (bo - 1) * s + 3, neighbouring tiles
// overlap by 3 - s pixels).  On the active output blocks
//     y = shortcut(x) + W3 ReLU(W2 *_s zero_outside(ReLU(W1 x + b1)) + b2) + b3,
// shortcut = a 1x1 convolution with the unit's stride (ws, bs) or the identity; other pixels of y stay.
//
// Shapes the one-kernel unit serves go to it: stride 1 with the identity shortcut, C in {64, 96, 128, 192, 256} (width
// a multiple of 8 up to 64) and C = 384 (width 72 .. 96), and stride 2 with a projected shortcut, Cin -> Cout in
// {64->96, 96->192, 192->256, 64->128, 128->256} (width up to 64) and 256->384 (width 72 .. 96); block sides multiples
// of 8, bf16 / f16.  Everything else runs as a sequence of the library's own calls on tile stacks in the caller's workspace,
// no kernel lives here:
//     gather (input tile) -> 1x1 + ReLU -> zero outside the image -> 3x3 with stride + ReLU -> 1x1
//     shortcut:  projection: the fused 1x1 convolution with stride writes y's active blocks;
//                identity:   the active blocks of x are copied to y (skipped when y is x);
//     scatter-add of the branch onto y.
// The sum therefore rounds the shortcut to the storage type before the branch is added (two roundings; the one-kernel
// forms add in fp32 and round once).
#include "common.h"

using namespace sbnet;

namespace {

size_t round256u(size_t v) { return (v + 255) / 256 * 256; }

struct UnitLayout {
    size_t x_off, t1_off, t2_off, t3_off, total;
};

bool unit_layout(sbnet_dtype dt, int cap, const sbnet_geom *g_in, const sbnet_geom *g_out, int Cin, int Cm, int Cout,
                 UnitLayout *l) {
    if (!is_float_dtype(dt) || cap < 0 || !geom_ok(g_in) || !geom_ok(g_out) || Cin <= 0 || Cm <= 0 || Cout <= 0) return false;
    const size_t es = (size_t)elem_bytes(dt);
    const size_t tin = (size_t)cap * g_in->bsize_h * g_in->bsize_w, tout = (size_t)cap * g_out->bsize_h * g_out->bsize_w;
    l->x_off = 0;
    l->t1_off = round256u(tin * Cin * es);
    l->t2_off = l->t1_off + round256u(tin * Cm * es);
    l->t3_off = l->t2_off + round256u(tout * Cm * es);
    l->total = l->t3_off + round256u(tout * (size_t)(Cout > Cin ? Cout : Cin) * es);     // t3, or the blocks of x on their way to y
    return true;
}

}  // namespace

extern "C" size_t sbnet_sparse_unit_workspace_bytes(sbnet_dtype dtype, int cap, const sbnet_geom *g_in,
                                                    const sbnet_geom *g_out, int Cin, int Cm, int Cout) {
    UnitLayout l;
    return unit_layout(dtype, cap, g_in, g_out, Cin, Cm, Cout, &l) ? l.total : 0;
}

extern "C" sbnet_status sbnet_sparse_unit(const void *x, sbnet_dtype dtype, int N, int H, int W, int Cin, int Cm, int Cout,
                                          int stride, const int32_t *indices, const int32_t *count, int cap,
                                          const sbnet_geom *g_in, const sbnet_geom *g_out, const void *w1, const float *b1,
                                          const void *w2, const float *b2, const void *w3, const float *b3,
                                          const void *w_shortcut, const float *b_shortcut, void *y, int H_out, int W_out,
                                          void *workspace, size_t workspace_bytes, void *stream) {
    const char *who = "sbnet_sparse_unit";
    if (!x || !y || !indices || !count || !w1 || !w2 || !w3 || !b1 || !b2 || !b3)
        return fail(SBNET_EINVAL, "%s: null pointer (biases are required)", who);
    if (N <= 0 || H <= 0 || W <= 0 || H_out <= 0 || W_out <= 0 || Cin <= 0 || Cm <= 0 || Cout <= 0 || cap < 0 || stride <= 0)
        return fail(SBNET_EINVAL, "%s: bad sizes", who);
    if (!geom_ok(g_in) || !geom_ok(g_out)) return fail(SBNET_EINVAL, "%s: bad geometry", who);
    if ((g_in->bsize_h - 3) / stride + 1 != g_out->bsize_h || (g_in->bsize_w - 3) / stride + 1 != g_out->bsize_w ||
        g_in->boffset_h != -1 || g_in->boffset_w != -1 || g_in->bstride_h != g_out->bsize_h * stride ||
        g_in->bstride_w != g_out->bsize_w * stride || g_out->bstride_h != g_out->bsize_h || g_out->bstride_w != g_out->bsize_w ||
        g_out->boffset_h != 0 || g_out->boffset_w != 0 || g_in->bcount_h != g_out->bcount_h || g_in->bcount_w != g_out->bcount_w)
        return fail(SBNET_EINVAL, "%s: g_in / g_out must be the geometries of a 3x3 convolution with this stride", who);
    if (!w_shortcut && (Cin != Cout || stride != 1))
        return fail(SBNET_EINVAL, "%s: the identity shortcut needs stride 1 and equal channel counts", who);
    if (w_shortcut && !b_shortcut) return fail(SBNET_EINVAL, "%s: a projected shortcut needs its bias", who);
    if (is_float_dtype(dtype) && x != y &&
        ranges_overlap(x, (size_t)N * H * W * Cin * elem_bytes(dtype), y, (size_t)N * H_out * W_out * Cout * elem_bytes(dtype)))
        return fail(SBNET_EINVAL, "%s: y must be x itself (identity shortcut only) or not overlap it", who);
    if (w_shortcut && x == y) return fail(SBNET_EINVAL, "%s: y must not alias x with a projected shortcut", who);
    if (cap == 0) return SBNET_OK;

    // the one-kernel unit where it applies (it needs two buffers)
    if (!w_shortcut && x != y) {
        sbnet_status st = sbnet_sparse_bottleneck(x, dtype, N, H, W, Cin, Cm, indices, count, cap, g_in, g_out, w1, b1, w2, b2,
                                                  w3, b3, y, stream);
        if (st != SBNET_EUNSUPPORTED) return st;
    }

    // ... and the one-kernel downsampling unit
    if (w_shortcut && stride == 2) {
        sbnet_status st = unit_down_try(who, x, dtype, N, H, W, Cin, Cm, Cout, indices, count, cap, g_in, g_out, w1, b1, w2, b2,
                                        w3, b3, w_shortcut, b_shortcut, y, H_out, W_out, stream);
        if (st != SBNET_EUNSUPPORTED) return st;
    }

    UnitLayout l;
    if (!unit_layout(dtype, cap, g_in, g_out, Cin, Cm, Cout, &l)) return fail(SBNET_EUNSUPPORTED, "%s: dtype must be f32, bf16 or f16", who);
    if (!workspace || workspace_bytes < l.total || ((uintptr_t)workspace & 255))
        return fail(SBNET_EINVAL, "%s: workspace of %zu bytes, 256-byte aligned, needed for this shape", who, l.total);
    unsigned char *ws = (unsigned char *)workspace;
    void *tx = ws + l.x_off, *t1 = ws + l.t1_off, *t2 = ws + l.t2_off, *t3 = ws + l.t3_off;
    const int th = g_in->bsize_h, tw = g_in->bsize_w, oh = g_out->bsize_h, ow = g_out->bsize_w;
    sbnet_status st;
#define SBNET_STEP(call) do { st = (call); if (st != SBNET_OK) return st; } while (0)
    SBNET_STEP(sbnet_sparse_gather(x, dtype, N, H, W, Cin, indices, count, cap, g_in, tx, stream));
    SBNET_STEP(sbnet_conv_on_tiles(tx, dtype, count, cap, th, tw, Cin, w1, b1, 1, 1, 1, 1, Cm, 1, t1, stream));
    SBNET_STEP(sbnet_zero_outside(t1, dtype, H, W, Cm, indices, count, cap, g_in, stream));
    SBNET_STEP(sbnet_conv_on_tiles(t1, dtype, count, cap, th, tw, Cm, w2, b2, 3, 3, stride, stride, Cm, 1, t2, stream));
    if (w_shortcut) {
        // the shortcut first: it writes the active blocks of y; the branch is then added onto them
        sbnet_geom g_sc = *g_out;            // input side of a 1x1 convolution with this stride
        g_sc.bsize_h = (oh - 1) * stride + 1; g_sc.bsize_w = (ow - 1) * stride + 1;
        g_sc.bstride_h = oh * stride; g_sc.bstride_w = ow * stride;
        SBNET_STEP(sbnet_sparse_conv(x, dtype, N, H, W, Cin, indices, count, cap, &g_sc, g_out, w_shortcut, b_shortcut, 1, 1,
                                     stride, stride, Cout, 0, y, H_out, W_out, 0, stream));
    } else if (x != y) {
        SBNET_STEP(sbnet_sparse_gather(x, dtype, N, H, W, Cin, indices, count, cap, g_out, t3, stream));
        SBNET_STEP(sbnet_sparse_scatter(t3, dtype, indices, count, cap, g_out, y, N, H_out, W_out, Cout, 0, stream));
    }
    SBNET_STEP(sbnet_conv_on_tiles(t2, dtype, count, cap, oh, ow, Cm, w3, b3, 1, 1, 1, 1, Cout, 0, t3, stream));
    SBNET_STEP(sbnet_sparse_scatter(t3, dtype, indices, count, cap, g_out, y, N, H_out, W_out, Cout, 1, stream));
#undef SBNET_STEP
    return SBNET_OK;
}
