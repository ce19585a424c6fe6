// Training forward and backward of the residual branch of a sparse bottleneck unit on tiles (Sec. 3.3 of arXiv 1801.02108; training
// is the subject of the section's last paragraph), as a composition of the library's own calls: no kernel lives here.
// With the forward pass  t1 = zero_outside(ReLU(W1 x + b1)),  t2 = ReLU(W2 * t1 + b2),  t3 = W3 t2 + b3  kept by the
// caller (the fused forward kernel does not keep t1 and t2; a training forward runs the three convolutions as
// single calls), and dt3 = dL/dt3 given:
//   dW3 = t2^T dt3,  db3 = sum dt3,  dt2 = (dt3 W3^T) where t2 > 0
//   dW2 = corr(t1, dt2),  db2 = sum dt2,  dt1 = (dt2 * W2 mirrored) where t1 > 0   (t1 = 0 outside the image, so its
//                                                                              mask also blocks the gradient there)
//   dW1 = x^T dt1,  db1 = sum dt1,  dx = dt1 W1^T
// Every step is one of sbnet_conv_on_tiles_backward_weights / _backward_data, sbnet_bias_backward_on_tiles and
// sbnet_relu_bias_backward_on_tiles (the ReLU mask and the bias sum of the masked gradient in one pass); the workspace
// holds dt2, dt1 and the largest scratch any of them asks for.
// The matching forward pass that keeps t1 and t2 is the same three convolutions as single calls plus the zeroing of
// t1 outside the image.
#include "common.h"

using namespace sbnet;

namespace {

struct BwdLayout {
    size_t dt2_off, dt1_off, scratch_off, scratch_bytes, total;
};

size_t round256(size_t v) { return (v + 255) / 256 * 256; }

bool layout_of(sbnet_dtype dt, int cap, int th, int tw, int oh, int ow, int C, int Cm, BwdLayout *l) {
    if (!is_float_dtype(dt) || cap < 0 || th < 3 || tw < 3 || oh != th - 2 || ow != tw - 2 || C <= 0 || Cm <= 0) return false;
    const size_t es = (size_t)elem_bytes(dt);
    l->dt2_off = 0;
    l->dt1_off = round256((size_t)cap * oh * ow * Cm * es);
    l->scratch_off = l->dt1_off + round256((size_t)cap * th * tw * Cm * es);
    size_t s = 0;
    auto need = [&](size_t v) { if (v > s) s = v; };
    need(sbnet_conv_backward_weights_workspace_bytes(dt, cap, oh, ow, Cm, 1, 1, 1, 1, C));      // dW3
    need(sbnet_conv_backward_weights_workspace_bytes(dt, cap, th, tw, Cm, 3, 3, 1, 1, Cm));     // dW2
    need(sbnet_conv_backward_weights_workspace_bytes(dt, cap, th, tw, C, 1, 1, 1, 1, Cm));      // dW1
    need(sbnet_conv_backward_data_workspace_bytes(dt, cap, oh, ow, 1, 1, 1, 1, C));             // dt2
    need(sbnet_conv_backward_data_workspace_bytes(dt, cap, th, tw, 3, 3, 1, 1, Cm));            // dt1
    need(sbnet_conv_backward_data_workspace_bytes(dt, cap, th, tw, 1, 1, 1, 1, Cm));            // dx
    need(sbnet_bias_backward_workspace_bytes(cap, C));
    need(sbnet_bias_backward_workspace_bytes(cap, Cm));
    l->scratch_bytes = round256(s);
    l->total = l->scratch_off + l->scratch_bytes;
    return true;
}

}  // namespace

extern "C" size_t sbnet_bottleneck_backward_workspace_bytes(sbnet_dtype dtype, int cap, int th, int tw, int C, int Cm) {
    BwdLayout l;
    return layout_of(dtype, cap, th, tw, th - 2, tw - 2, C, Cm, &l) ? l.total : 0;
}

extern "C" sbnet_status sbnet_bottleneck_backward_on_tiles(const void *tiles_in, const void *t1, const void *t2, const void *dt3,
                                                           sbnet_dtype dtype, const int32_t *count, int cap, int th, int tw,
                                                           int C, int Cm, const void *w1_t, const void *w2_t, const void *w3_t,
                                                           void *dtiles_in, float *dw1, float *db1, float *dw2, float *db2,
                                                           float *dw3, float *db3, void *workspace, size_t workspace_bytes,
                                                           void *stream) {
    const char *who = "sbnet_bottleneck_backward_on_tiles";
    if (!tiles_in || !t1 || !t2 || !dt3 || !count || !w1_t || !w2_t || !w3_t || !dtiles_in || !dw1 || !db1 || !dw2 || !db2 ||
        !dw3 || !db3 || !workspace)
        return fail(SBNET_EINVAL, "%s: null pointer", who);
    BwdLayout l;
    if (!layout_of(dtype, cap, th, tw, th - 2, tw - 2, C, Cm, &l)) return fail(SBNET_EINVAL, "%s: bad sizes or dtype", who);
    if ((uintptr_t)workspace & 255) return fail(SBNET_EINVAL, "%s: workspace must be 256-byte aligned", who);
    if (workspace_bytes < l.total) return fail(SBNET_EINVAL, "%s: workspace too small", who);
    const int oh = th - 2, ow = tw - 2;
    char *ws = (char *)workspace;
    void *dt2 = ws + l.dt2_off, *dt1 = ws + l.dt1_off, *scratch = ws + l.scratch_off;
    const size_t sb = l.scratch_bytes;
    sbnet_status st;
#define SBNET_STEP(call)                 \
    do {                                 \
        st = (call);                     \
        if (st != SBNET_OK) return st;   \
    } while (0)
    // third convolution (1x1, Cm -> C)
    SBNET_STEP(sbnet_conv_on_tiles_backward_weights(t2, dt3, dtype, count, cap, oh, ow, Cm, 1, 1, 1, 1, C, dw3, scratch, sb, stream));
    SBNET_STEP(sbnet_bias_backward_on_tiles(dt3, dtype, count, cap, oh * ow, C, db3, scratch, sb, stream));
    SBNET_STEP(sbnet_conv_on_tiles_backward_data(dt3, dtype, count, cap, oh, ow, Cm, w3_t, 1, 1, 1, 1, C, dt2, scratch, sb, stream));
    SBNET_STEP(sbnet_relu_bias_backward_on_tiles(t2, dt2, dtype, count, cap, oh * ow, Cm, dt2, db2, scratch, sb, stream));
    // second convolution (3x3 valid, Cm -> Cm)
    SBNET_STEP(sbnet_conv_on_tiles_backward_weights(t1, dt2, dtype, count, cap, th, tw, Cm, 3, 3, 1, 1, Cm, dw2, scratch, sb, stream));
    SBNET_STEP(sbnet_conv_on_tiles_backward_data(dt2, dtype, count, cap, th, tw, Cm, w2_t, 3, 3, 1, 1, Cm, dt1, scratch, sb, stream));
    SBNET_STEP(sbnet_relu_bias_backward_on_tiles(t1, dt1, dtype, count, cap, th * tw, Cm, dt1, db1, scratch, sb, stream));
    // first convolution (1x1, C -> Cm)
    SBNET_STEP(sbnet_conv_on_tiles_backward_weights(tiles_in, dt1, dtype, count, cap, th, tw, C, 1, 1, 1, 1, Cm, dw1, scratch, sb, stream));
    SBNET_STEP(sbnet_conv_on_tiles_backward_data(dt1, dtype, count, cap, th, tw, C, w1_t, 1, 1, 1, 1, Cm, dtiles_in, scratch, sb, stream));
#undef SBNET_STEP
    return SBNET_OK;
}


extern "C" sbnet_status sbnet_bottleneck_forward_keep_on_tiles(const void *tiles_in, sbnet_dtype dtype, int H, int W, int C, int Cm,
                                                               const int32_t *indices, const int32_t *count, int cap,
                                                               const sbnet_geom *g_in, const void *w1, const float *b1,
                                                               const void *w2, const float *b2, const void *w3,
                                                               const float *b3, void *t1, void *t2, void *t3, void *stream) {
    const char *who = "sbnet_bottleneck_forward_keep_on_tiles";
    if (!tiles_in || !indices || !count || !g_in || !w1 || !w2 || !w3 || !t1 || !t2 || !t3)
        return fail(SBNET_EINVAL, "%s: null pointer", who);
    if (!geom_ok(g_in) || g_in->bsize_h < 3 || g_in->bsize_w < 3) return fail(SBNET_EINVAL, "%s: bad geometry", who);
    const int th = g_in->bsize_h, tw = g_in->bsize_w;
    sbnet_status st = sbnet_conv_on_tiles(tiles_in, dtype, count, cap, th, tw, C, w1, b1, 1, 1, 1, 1, Cm, 1, t1, stream);
    if (st != SBNET_OK) return st;
    st = sbnet_zero_outside(t1, dtype, H, W, Cm, indices, count, cap, g_in, stream);
    if (st != SBNET_OK) return st;
    st = sbnet_conv_on_tiles(t1, dtype, count, cap, th, tw, Cm, w2, b2, 3, 3, 1, 1, Cm, 1, t2, stream);
    if (st != SBNET_OK) return st;
    return sbnet_conv_on_tiles(t2, dtype, count, cap, th - 2, tw - 2, Cm, w3, b3, 1, 1, 1, 1, C, 0, t3, stream);
}
