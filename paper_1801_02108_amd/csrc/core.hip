// Host-only entry points: error text, block geometry (Sec. 3.1, Fig. 3 of arXiv 1801.02108)
// and the synchronising read-back of the active-block counter.
#include "common.h"

#include <mutex>

namespace sbnet {

static const sbnet_tuning kDefaultTuning = {3, 5, 8, 16};
static sbnet_tuning g_tuning = kDefaultTuning;
static std::mutex g_tuning_mutex;

sbnet_tuning tuning() {
    std::lock_guard<std::mutex> lock(g_tuning_mutex);
    return g_tuning;
}

char *error_buffer() {
    static thread_local char buf[512] = "";
    return buf;
}

sbnet_status fail(sbnet_status code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(error_buffer(), 512, fmt, ap);
    va_end(ap);
    return code;
}

}  // namespace sbnet

using namespace sbnet;

extern "C" const char *sbnet_last_error(void) { return error_buffer(); }

extern "C" sbnet_status sbnet_set_tuning(const sbnet_tuning *t) {
    if (t && (t->unit_small_item_cost_eighths < 0 || t->conv3_small_item_cost_eighths < 0 || t->wgrad_split_factor_3x3 < 1 ||
              t->wgrad_split_factor_1x1 < 1 || t->wgrad_split_factor_3x3 > 1024 || t->wgrad_split_factor_1x1 > 1024))
        return fail(SBNET_EINVAL, "sbnet_set_tuning: value out of range");
    std::lock_guard<std::mutex> lock(g_tuning_mutex);
    g_tuning = t ? *t : kDefaultTuning;
    return SBNET_OK;
}

extern "C" sbnet_status sbnet_get_tuning(sbnet_tuning *t) {
    if (!t) return fail(SBNET_EINVAL, "sbnet_get_tuning: null pointer");
    *t = tuning();
    return SBNET_OK;
}

extern "C" sbnet_status sbnet_geometry(int H, int W, int kh, int kw, int sh, int sw, int bo_h, int bo_w,
                                       sbnet_geom *g_in, sbnet_geom *g_out, int *H_out, int *W_out) {
    if (H <= 0 || W <= 0 || kh <= 0 || kw <= 0 || sh <= 0 || sw <= 0 || bo_h <= 0 || bo_w <= 0)
        return fail(SBNET_EINVAL, "sbnet_geometry: sizes must be positive");
    if (!g_in || !g_out) return fail(SBNET_EINVAL, "sbnet_geometry: null geometry pointer");
    int ph = (kh - 1) / 2, pw = (kw - 1) / 2;
    int Ho = (H + 2 * ph - kh) / sh + 1, Wo = (W + 2 * pw - kw) / sw + 1;
    if (Ho <= 0 || Wo <= 0) return fail(SBNET_EINVAL, "sbnet_geometry: empty output");
    int bh = (Ho + bo_h - 1) / bo_h, bw = (Wo + bo_w - 1) / bo_w;
    // input tile = receptive field of one output block; neighbours overlap by k - s pixels
    g_in->bsize_h = (bo_h - 1) * sh + kh;
    g_in->bsize_w = (bo_w - 1) * sw + kw;
    g_in->bstride_h = bo_h * sh;
    g_in->bstride_w = bo_w * sw;
    g_in->boffset_h = -ph;
    g_in->boffset_w = -pw;
    g_in->bcount_h = bh;
    g_in->bcount_w = bw;
    // output blocks tile the output without overlap
    g_out->bsize_h = g_out->bstride_h = bo_h;
    g_out->bsize_w = g_out->bstride_w = bo_w;
    g_out->boffset_h = g_out->boffset_w = 0;
    g_out->bcount_h = bh;
    g_out->bcount_w = bw;
    if (H_out) *H_out = Ho;
    if (W_out) *W_out = Wo;
    return SBNET_OK;
}

static int floor_div(int a, int b) { return a >= 0 ? a / b : -((-a + b - 1) / b); }

extern "C" sbnet_status sbnet_coarse_geometry(const sbnet_geom *g, int factor, sbnet_geom *coarse) {
    if (!g || !coarse) return fail(SBNET_EINVAL, "sbnet_coarse_geometry: null geometry pointer");
    if (factor <= 0 || g->bsize_h <= 0 || g->bsize_w <= 0 || g->bstride_h <= 0 || g->bstride_w <= 0)
        return fail(SBNET_EINVAL, "sbnet_coarse_geometry: sizes must be positive");
    if (g->bstride_h % factor || g->bstride_w % factor)
        return fail(SBNET_EINVAL, "sbnet_coarse_geometry: the block stride must be a multiple of the factor");
    // window b covers pixels [o + b S, o + b S + B): the cells floor(first / f) .. floor(last / f); S is a multiple
    // of f, so the count of cells is the same for every b
    coarse->boffset_h = floor_div(g->boffset_h, factor);
    coarse->boffset_w = floor_div(g->boffset_w, factor);
    coarse->bsize_h = floor_div(g->boffset_h + g->bsize_h - 1, factor) - coarse->boffset_h + 1;
    coarse->bsize_w = floor_div(g->boffset_w + g->bsize_w - 1, factor) - coarse->boffset_w + 1;
    coarse->bstride_h = g->bstride_h / factor;
    coarse->bstride_w = g->bstride_w / factor;
    coarse->bcount_h = g->bcount_h;
    coarse->bcount_w = g->bcount_w;
    return SBNET_OK;
}

extern "C" sbnet_status sbnet_read_count(const int32_t *count, int cap, int *host_count, void *stream) {
    if (!count || !host_count) return fail(SBNET_EINVAL, "sbnet_read_count: null pointer");
    int32_t v = 0;
    hipError_t e = hipMemcpyAsync(&v, count, sizeof(v), hipMemcpyDeviceToHost, (hipStream_t)stream);
    if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess) return fail(SBNET_EHIP, "sbnet_read_count: %s", hipGetErrorString(e));
    *host_count = v;
    if (v > cap) return fail(SBNET_ECAP, "sbnet_read_count: %d active blocks exceed cap %d", v, cap);
    return SBNET_OK;
}
