// Transposing gather / scatter / scatter-add (Sec. 3.4 of arXiv 1801.02108, "Fused transpose+gather and
// transpose+scatter kernels"): the feature map stays NHWC, where a strip of w x C elements is contiguous, and the
// tile stack is channel-major, [B][C][h][w], for a consumer that wants that layout; the transpose rides along with
// the copy instead of costing a round trip through memory of its own.  (The matrix-core kernels of this library
// consume NHWC tiles and use the plain copies of gather_scatter.hip; these entry points serve other consumers.)
//
// One work item is (active block, slab of 128 bytes of channels per pixel: 64 two-byte or 32 four-byte channels).
// The slab passes through LDS in the tile stack's own order, [channel][pixel], without padding, so that the tile
// side of the copy is a straight run of 16-byte vectors (a slab of a tile is contiguous in the stack); the NHWC side
// moves 16-byte vectors of neighbouring channels, eight lanes per 128-byte pixel strip, and the element-wise
// transposition happens between registers and LDS with narrow LDS accesses.  When a channel row of the slab is a
// whole number of 16-byte vectors (h*w % 8 == 0 for two-byte elements), rows can start in the same bank (256 pixels:
// every row does) and the eight lanes that hold one pixel's channel groups would collide 16-way; the vectors of
// channel c are therefore rotated inside their row by c / 8 places, which spreads those lanes over the banks and
// keeps the tile side a permuted run of whole vectors.
#include "tile_add.h"

namespace sbnet {

constexpr int kTThreads = 256;
constexpr int kTUnroll = 4;
constexpr int kTLdsMax = 160 * 1024;

struct TCopyParams {
    sbnet_geom g;
    int H, W, C, cap;
    int hw;                  // pixels per tile
    int slabs;               // slabs per tile
    int cs;                  // channels per full slab
    int vpp_last;            // 16-byte vectors per pixel in the last slab (C need not be a multiple of cs)
    int row_vecs;            // 16-byte vectors per channel row of the slab when rows are whole vectors, else 0 (no rotation)
    FastDiv div_slabs, div_w, div_vpp, div_vpp_last, div_rv;
};

template <int ES> struct TElem;
template <> struct TElem<2> { typedef uint16_t T; };
template <> struct TElem<4> { typedef uint32_t T; };

template <int ES>
__device__ __forceinline__ typename TElem<ES>::T vec_elem(const uint4 &v, int e) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    if (ES == 4) return (typename TElem<ES>::T)w[e];
    return (typename TElem<ES>::T)(w[e >> 1] >> ((e & 1) * 16));
}
template <int ES>
__device__ __forceinline__ uint4 vec_from(const typename TElem<ES>::T *el) {
    if (ES == 4) return make_uint4(el[0], el[1], el[2], el[3]);
    return make_uint4((uint32_t)el[0] | ((uint32_t)el[1] << 16), (uint32_t)el[2] | ((uint32_t)el[3] << 16),
                      (uint32_t)el[4] | ((uint32_t)el[5] << 16), (uint32_t)el[6] | ((uint32_t)el[7] << 16));
}

// MODE 0: gather (image -> tiles, zero fill), 1: scatter (tiles -> image), 2: scatter-add.
template <int ES, int MODE, int DT>
__global__ __launch_bounds__(kTThreads) void tile_transpose(uint4 *__restrict__ img, uint4 *__restrict__ tiles,
                                                            const int32_t *__restrict__ indices,
                                                            const int32_t *__restrict__ count, TCopyParams p) {
    typedef typename TElem<ES>::T E;
    constexpr int EPV = 16 / ES;                                  // elements per 16-byte vector
    extern __shared__ __align__(16) unsigned char lds[];          // [channel of the slab][pixel]
    E *le = (E *)lds;
    uint4 *lv = (uint4 *)lds;
    const int nact = min(*count, p.cap);
    const uint32_t items = (uint32_t)nact * (uint32_t)p.slabs;
    const uint32_t pix_vecs = (uint32_t)p.C / EPV;                // vectors per pixel of the image
    for (uint32_t item = blockIdx.x; item < items; item += gridDim.x) {
        const uint32_t b = fdiv(item, p.div_slabs);
        const int slab = (int)(item - b * p.slabs);
        const bool last = slab == p.slabs - 1;
        const uint32_t vpp = last ? (uint32_t)p.vpp_last : (uint32_t)(p.cs / EPV);       // vectors per pixel in this slab
        const FastDiv dvpp = last ? p.div_vpp_last : p.div_vpp;
        const uint32_t nvec = (uint32_t)p.hw * vpp;               // vectors of the slab, on either side
        const int n = indices[3 * b], by = indices[3 * b + 1], bx = indices[3 * b + 2];
        const int y0 = p.g.boffset_h + by * p.g.bstride_h;
        const int x0 = p.g.boffset_w + bx * p.g.bstride_w;
        // a slab of a tile is contiguous in the channel-major stack
        uint4 *tile = tiles + ((size_t)b * p.C + (size_t)slab * p.cs) * p.hw / EPV;
        const long long img_base = (long long)n * p.H * p.W * pix_vecs + (long long)slab * (p.cs / EPV);
        // image-side vector v: pixel v / vpp of the tile, vector v % vpp of the slab's channels
        auto locate = [&](uint32_t v, uint32_t &px, uint32_t &k, long long &src) __attribute__((always_inline)) {
            px = fdiv(v, dvpp);
            k = v - px * vpp;
            const uint32_t i = fdiv(px, p.div_w), j = px - i * p.g.bsize_w;
            const int yy = y0 + (int)i, xx = x0 + (int)j;
            src = img_base + ((long long)yy * p.W + xx) * pix_vecs + k;
            return v < nvec && yy >= 0 && yy < p.H && xx >= 0 && xx < p.W;
        };
        // LDS position of element (channel ch of the slab, pixel px), and of tile-side vector v
        auto lds_elem = [&](uint32_t ch, uint32_t px) __attribute__((always_inline)) {
            if (p.row_vecs == 0) return ch * (uint32_t)p.hw + px;
            uint32_t pg = px / EPV + ch / EPV;                    // rotate by the channel's vector number
            pg = pg >= (uint32_t)p.row_vecs ? pg - (uint32_t)p.row_vecs : pg;
            pg = pg >= (uint32_t)p.row_vecs ? pg - (uint32_t)p.row_vecs : pg;
            return ch * (uint32_t)p.hw + pg * EPV + px % EPV;
        };
        auto lds_vec = [&](uint32_t v) __attribute__((always_inline)) {
            if (p.row_vecs == 0) return v;
            const uint32_t ch = fdiv(v, p.div_rv);
            uint32_t pg = v - ch * (uint32_t)p.row_vecs + ch / EPV;
            pg = pg >= (uint32_t)p.row_vecs ? pg - (uint32_t)p.row_vecs : pg;
            pg = pg >= (uint32_t)p.row_vecs ? pg - (uint32_t)p.row_vecs : pg;
            return ch * (uint32_t)p.row_vecs + pg;
        };
        if (MODE == 0) {
            for (uint32_t v0 = threadIdx.x; v0 < nvec; v0 += kTThreads * kTUnroll) {
                uint4 val[kTUnroll];
                uint32_t px[kTUnroll], k[kTUnroll];
#pragma unroll
                for (int u = 0; u < kTUnroll; ++u) {
                    long long src;
                    const bool inside = locate(v0 + u * kTThreads, px[u], k[u], src);
                    val[u] = make_uint4(0, 0, 0, 0);
                    if (inside) val[u] = img[src];
                }
#pragma unroll
                for (int u = 0; u < kTUnroll; ++u)
                    if (v0 + u * kTThreads < nvec) {
#pragma unroll
                        for (int e = 0; e < EPV; ++e) le[lds_elem(k[u] * EPV + e, px[u])] = vec_elem<ES>(val[u], e);
                    }
            }
            __syncthreads();
            for (uint32_t v = threadIdx.x; v < nvec; v += kTThreads) tile[v] = lv[lds_vec(v)];
        } else {
            for (uint32_t v0 = threadIdx.x; v0 < nvec; v0 += kTThreads * kTUnroll) {
                uint4 val[kTUnroll];
#pragma unroll
                for (int u = 0; u < kTUnroll; ++u) {
                    val[u] = make_uint4(0, 0, 0, 0);
                    if (v0 + u * kTThreads < nvec) val[u] = tile[v0 + u * kTThreads];
                }
#pragma unroll
                for (int u = 0; u < kTUnroll; ++u)
                    if (v0 + u * kTThreads < nvec) lv[lds_vec(v0 + u * kTThreads)] = val[u];
            }
            __syncthreads();
            for (uint32_t v0 = threadIdx.x; v0 < nvec; v0 += kTThreads * kTUnroll) {
                uint4 val[kTUnroll], old[kTUnroll];
                long long src[kTUnroll];
                bool inside[kTUnroll];
#pragma unroll
                for (int u = 0; u < kTUnroll; ++u) {
                    uint32_t px, k;
                    inside[u] = locate(v0 + u * kTThreads, px, k, src[u]);
                    old[u] = make_uint4(0, 0, 0, 0);
                    if (MODE == 2 && inside[u]) old[u] = img[src[u]];
                    E el[EPV];
#pragma unroll
                    for (int e = 0; e < EPV; ++e) el[e] = inside[u] ? le[lds_elem(k * EPV + e, px)] : (E)0;
                    val[u] = vec_from<ES>(el);
                }
#pragma unroll
                for (int u = 0; u < kTUnroll; ++u)
                    if (inside[u]) {
                        if (MODE == 2)
                            val[u] = make_uint4(add_word<DT>(old[u].x, val[u].x), add_word<DT>(old[u].y, val[u].y),
                                                add_word<DT>(old[u].z, val[u].z), add_word<DT>(old[u].w, val[u].w));
                        img[src[u]] = val[u];
                    }
            }
        }
        __syncthreads();                                          // LDS free for the next item
    }
}

template <int ES, int MODE, int DT>
static void launch_t(void *img, void *tiles, const int32_t *indices, const int32_t *count, const TCopyParams &p,
                     size_t lds_bytes, hipStream_t s) {
    const long long items = (long long)p.cap * p.slabs;
    const int grid = (int)(items < 4096 ? items : 4096);
    auto kern = tile_transpose<ES, MODE, DT>;
    if (lds_bytes > 48 * 1024)
        (void)hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kTThreads), lds_bytes, s, (uint4 *)img, (uint4 *)tiles, indices, count, p);
}

static sbnet_status transpose_entry(const char *who, int mode, void *img, void *tiles, sbnet_dtype dt, int N, int H,
                                    int W, int C, const int32_t *indices, const int32_t *count, int cap,
                                    const sbnet_geom *g, void *stream) {
    if (!img || !tiles || !indices || !count) return fail(SBNET_EINVAL, "%s: null pointer", who);
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || cap < 0) return fail(SBNET_EINVAL, "%s: bad sizes", who);
    if (!geom_ok(g)) return fail(SBNET_EINVAL, "%s: bad geometry", who);
    if (!is_float_dtype(dt)) return fail(SBNET_EUNSUPPORTED, "%s: dtype must be f32, bf16 or f16", who);
    if (mode != 0 && (g->bstride_h < g->bsize_h || g->bstride_w < g->bsize_w))
        return fail(SBNET_EINVAL, "%s: scatter needs non-overlapping blocks (bstride >= bsize)", who);
    if (((uintptr_t)img | (uintptr_t)tiles) & 15) return fail(SBNET_EINVAL, "%s: pointers must be 16-byte aligned", who);
    const int es = elem_bytes(dt);
    if ((long long)C * es % 16) return fail(SBNET_EUNSUPPORTED, "%s: a pixel's channels must fill 16-byte vectors", who);
    const long long hw = (long long)g->bsize_h * g->bsize_w;
    const size_t lds_bytes = (size_t)(128 * hw);                  // a slab: 128 bytes of channels for every pixel
    if (lds_bytes > (size_t)kTLdsMax) return fail(SBNET_EUNSUPPORTED, "%s: tiles above 1280 pixels are not supported", who);
    if (cap == 0) return SBNET_OK;
    TCopyParams p;
    p.g = *g;
    p.H = H; p.W = W; p.C = C; p.cap = cap;
    p.hw = (int)hw;
    p.cs = 128 / es;
    p.slabs = (C + p.cs - 1) / p.cs;
    p.vpp_last = (C - (p.slabs - 1) * p.cs) * es / 16;
    if ((long long)cap * p.slabs >= (1LL << 31) || (long long)N * H * W * C * es / 16 >= (1LL << 40))
        return fail(SBNET_EUNSUPPORTED, "%s: tensor too large", who);
    p.div_slabs = make_fastdiv((uint32_t)p.slabs);
    p.div_w = make_fastdiv((uint32_t)g->bsize_w);
    p.div_vpp = make_fastdiv(8u);
    p.div_vpp_last = make_fastdiv((uint32_t)p.vpp_last);
    // rotation needs whole vectors per row and at least as many of them as the largest shift (cs / EPV - 1 = 7) twice over
    p.row_vecs = (hw * es % 16 == 0 && hw * es / 16 >= 8) ? (int)(hw * es / 16) : 0;
    p.div_rv = make_fastdiv((uint32_t)(p.row_vecs ? p.row_vecs : 1));
    hipStream_t s = (hipStream_t)stream;
#define SBNET_T(MODE)                                                                                                 \
    do {                                                                                                              \
        if (dt == SBNET_F32) launch_t<4, MODE, SBNET_F32>(img, tiles, indices, count, p, lds_bytes, s);               \
        else if (dt == SBNET_BF16) launch_t<2, MODE, SBNET_BF16>(img, tiles, indices, count, p, lds_bytes, s);        \
        else launch_t<2, MODE, SBNET_F16>(img, tiles, indices, count, p, lds_bytes, s);                               \
    } while (0)
    if (mode == 0) SBNET_T(0);
    else if (mode == 1) SBNET_T(1);
    else SBNET_T(2);
#undef SBNET_T
    return launch_status(who);
}

}  // namespace sbnet

using namespace sbnet;

extern "C" sbnet_status sbnet_sparse_gather_chw(const void *x, sbnet_dtype dtype, int N, int H, int W, int C,
                                                const int32_t *indices, const int32_t *count, int cap,
                                                const sbnet_geom *g, void *tiles_chw, void *stream) {
    return transpose_entry("sbnet_sparse_gather_chw", 0, const_cast<void *>(x), tiles_chw, dtype, N, H, W, C, indices,
                           count, cap, g, stream);
}

extern "C" sbnet_status sbnet_sparse_scatter_chw(const void *tiles_chw, sbnet_dtype dtype, const int32_t *indices,
                                                 const int32_t *count, int cap, const sbnet_geom *g, void *y, int N,
                                                 int H, int W, int C, int add, void *stream) {
    return transpose_entry("sbnet_sparse_scatter_chw", add ? 2 : 1, y, const_cast<void *>(tiles_chw), dtype, N, H, W, C,
                           indices, count, cap, g, stream);
}
