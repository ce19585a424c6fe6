// sparse_gather / sparse_scatter / scatter-add (Sec. 3.2 "Gather kernel", "Scatter kernel" and
// Sec. 3.4 "Fused scatter-add kernel for residual blocks" of arXiv 1801.02108).
//
// Both directions are one HBM-bound copy between an NHWC feature map and a [B][h][w][C] tile
// stack.  The paper fuses an NHWC->NCHW transpose into these kernels because its dense library
// wanted NCHW; the MFMA convolution here consumes NHWC, so a tile row (w*C elements) stays one
// contiguous strip on both sides and is moved with the widest vector the channel count allows.
//
// Work decomposition: a tile is cut into S segments of consecutive vectors; workgroups stride
// over (tile, segment) items and stop at the device-side active count, so the launch does not
// depend on a host read-back of that count.
#include "tile_add.h"

namespace sbnet {

constexpr int kCopyThreads = 256;
constexpr int kCopyUnroll = 4;

struct CopyParams {
    sbnet_geom g;
    int H, W;
    int cap;
    int segs;             // segments per tile
    uint32_t tile_vecs;   // vectors per tile
    uint32_t seg_vecs;    // vectors per segment (last one may be shorter)
    uint32_t row_vecs;    // vectors per tile row  = bsize_w * pix_vecs
    uint32_t pix_vecs;    // vectors per pixel     = C * elem_bytes / sizeof(V)
    FastDiv div_row;
    FastDiv div_segs;
};

template <int DT> __device__ __forceinline__ uint4 vadd(uint4 y, uint4 t) {
    return make_uint4(add_word<DT>(y.x, t.x), add_word<DT>(y.y, t.y), add_word<DT>(y.z, t.z), add_word<DT>(y.w, t.w));
}
template <int DT> __device__ __forceinline__ uint2 vadd(uint2 y, uint2 t) {
    return make_uint2(add_word<DT>(y.x, t.x), add_word<DT>(y.y, t.y));
}
template <int DT> __device__ __forceinline__ uint32_t vadd(uint32_t y, uint32_t t) { return add_word<DT>(y, t); }
template <int DT> __device__ __forceinline__ uint16_t vadd(uint16_t y, uint16_t t) {
    if (DT == SBNET_BF16) return (uint16_t)float_to_bf16_bits(bf16_bits_to_float(y) + bf16_bits_to_float(t));
    return (uint16_t)f16_add_bits(y, t);
}

__device__ __forceinline__ void vzero(uint4 &v) { v = make_uint4(0, 0, 0, 0); }
__device__ __forceinline__ void vzero(uint2 &v) { v = make_uint2(0, 0); }
__device__ __forceinline__ void vzero(uint32_t &v) { v = 0; }
__device__ __forceinline__ void vzero(uint16_t &v) { v = 0; }

// MODE 0: gather (image -> tiles, zero fill), 1: scatter (tiles -> image), 2: scatter-add,
// 3: zero the tile positions that lie outside the image (img is not touched).
template <typename V, int MODE, int DT>
__global__ __launch_bounds__(kCopyThreads) void tile_copy(V *__restrict__ img, V *__restrict__ tiles,
                                                           const int32_t *__restrict__ indices,
                                                           const int32_t *__restrict__ count, CopyParams p) {
    const int nact = min(*count, p.cap);
    const uint32_t items = (uint32_t)nact * (uint32_t)p.segs;
    for (uint32_t item = blockIdx.x; item < items; item += gridDim.x) {
        const uint32_t b = fdiv(item, p.div_segs);
        const uint32_t seg = item - b * p.segs;
        const int n = indices[3 * b], by = indices[3 * b + 1], bx = indices[3 * b + 2];
        const int y0 = p.g.boffset_h + by * p.g.bstride_h;
        const int x0 = p.g.boffset_w + bx * p.g.bstride_w;
        // columns of the tile that fall inside the image, in vector units of one tile row
        const uint32_t rem_lo = (uint32_t)max(0, -x0) * p.pix_vecs;
        const uint32_t rem_hi = (uint32_t)max(0, min(p.g.bsize_w, p.W - x0)) * p.pix_vecs;
        const uint32_t v_end = min(p.tile_vecs, (seg + 1) * p.seg_vecs);
        V *tile = tiles + (size_t)b * p.tile_vecs;
        const long long img_base = ((long long)n * p.H * p.W + x0) * (long long)p.pix_vecs;

        for (uint32_t v0 = seg * p.seg_vecs + threadIdx.x; v0 < v_end; v0 += kCopyThreads * kCopyUnroll) {
            V val[kCopyUnroll];
            long long src[kCopyUnroll];
            bool inside[kCopyUnroll], live[kCopyUnroll];
#pragma unroll
            for (int u = 0; u < kCopyUnroll; ++u) {
                const uint32_t v = v0 + u * kCopyThreads;
                live[u] = v < v_end;
                const uint32_t i = fdiv(v, p.div_row);
                const uint32_t rem = v - i * p.row_vecs;
                const int yy = y0 + (int)i;
                inside[u] = live[u] && yy >= 0 && yy < p.H && rem >= rem_lo && rem < rem_hi;
                src[u] = img_base + (long long)yy * p.W * p.pix_vecs + rem;
            }
            if (MODE == 3) {
#pragma unroll
                for (int u = 0; u < kCopyUnroll; ++u) {
                    vzero(val[u]);
                    if (live[u] && !inside[u]) tile[v0 + u * kCopyThreads] = val[u];
                }
            } else if (MODE == 0) {
#pragma unroll
                for (int u = 0; u < kCopyUnroll; ++u) {
                    vzero(val[u]);
                    if (inside[u]) val[u] = img[src[u]];
                }
#pragma unroll
                for (int u = 0; u < kCopyUnroll; ++u)
                    if (live[u]) tile[v0 + u * kCopyThreads] = val[u];
            } else {
                // tile reads depend only on `live`, so all of them are issued before any store
#pragma unroll
                for (int u = 0; u < kCopyUnroll; ++u) {
                    vzero(val[u]);
                    if (live[u]) val[u] = tile[v0 + u * kCopyThreads];
                }
                if (MODE == 2) {
                    V old[kCopyUnroll];
#pragma unroll
                    for (int u = 0; u < kCopyUnroll; ++u) {
                        vzero(old[u]);
                        if (inside[u]) old[u] = img[src[u]];
                    }
#pragma unroll
                    for (int u = 0; u < kCopyUnroll; ++u)
                        if (inside[u]) val[u] = vadd<DT>(old[u], val[u]);
                }
#pragma unroll
                for (int u = 0; u < kCopyUnroll; ++u)
                    if (inside[u]) img[src[u]] = val[u];
            }
        }
    }
}

template <typename V, int MODE, int DT>
static void launch_copy(void *img, void *tiles, const int32_t *indices, const int32_t *count,
                        const CopyParams &p, hipStream_t s) {
    long long items = (long long)p.cap * p.segs;
    int grid = (int)(items < 16384 ? (items > 0 ? items : 1) : 16384);
    hipLaunchKernelGGL((tile_copy<V, MODE, DT>), dim3(grid), dim3(kCopyThreads), 0, s, (V *)img, (V *)tiles,
                       indices, count, p);
}

template <int MODE, int DT>
static sbnet_status dispatch_vec(int vec_bytes, void *img, void *tiles, const int32_t *indices,
                                 const int32_t *count, const CopyParams &p, hipStream_t s) {
    switch (vec_bytes) {
        case 16: launch_copy<uint4, MODE, DT>(img, tiles, indices, count, p, s); break;
        case 8: launch_copy<uint2, MODE, DT>(img, tiles, indices, count, p, s); break;
        case 4: launch_copy<uint32_t, MODE, DT>(img, tiles, indices, count, p, s); break;
        case 2:
            if (DT == SBNET_F32) return fail(SBNET_EINVAL, "tile copy: 2-byte vectors with f32 data");
            launch_copy<uint16_t, MODE, (DT == SBNET_F32 ? SBNET_BF16 : DT)>(img, tiles, indices, count, p, s);
            break;
        default: return fail(SBNET_EINVAL, "tile copy: bad vector width");
    }
    return launch_status("tile copy");
}

static sbnet_status tile_copy_entry(const char *who, int mode, void *img, void *tiles, sbnet_dtype dt, int N,
                                    int H, int W, int C, const int32_t *indices, const int32_t *count, int cap,
                                    const sbnet_geom *g, void *stream) {
    if (!img || !tiles || !indices || !count) return fail(SBNET_EINVAL, "%s: null pointer", who);
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || cap < 0) return fail(SBNET_EINVAL, "%s: bad sizes", who);
    if (!geom_ok(g)) return fail(SBNET_EINVAL, "%s: bad geometry", who);
    if (!is_float_dtype(dt)) return fail(SBNET_EUNSUPPORTED, "%s: dtype must be f32, bf16 or f16", who);
    if ((mode == 1 || mode == 2) && (g->bstride_h < g->bsize_h || g->bstride_w < g->bsize_w))
        return fail(SBNET_EINVAL, "%s: scatter needs non-overlapping blocks (bstride >= bsize)", who);
    if (((uintptr_t)img | (uintptr_t)tiles) & 15) return fail(SBNET_EINVAL, "%s: pointers must be 16-byte aligned", who);
    if (cap == 0) return SBNET_OK;

    const long long pix_bytes = (long long)C * elem_bytes(dt);
    int vec = 16;
    while (pix_bytes % vec) vec >>= 1;
    const long long pix_vecs = pix_bytes / vec;
    const long long row_vecs = pix_vecs * g->bsize_w;
    const long long tile_vecs = row_vecs * g->bsize_h;
    const long long img_vecs = (long long)N * H * W * pix_vecs;
    if (tile_vecs >= (1LL << 31) || img_vecs >= (1LL << 40) || (long long)cap * 3 >= (1LL << 31))
        return fail(SBNET_EUNSUPPORTED, "%s: tensor too large", who);

    CopyParams p;
    p.g = *g;
    p.H = H;
    p.W = W;
    p.cap = cap;
    // segments of about 2048 vectors: enough workgroups to fill 256 CUs even with few tiles
    long long segs = (tile_vecs + 2047) / 2048;
    if (segs * cap >= (1LL << 31)) return fail(SBNET_EUNSUPPORTED, "%s: too many work items", who);
    p.segs = (int)segs;
    p.tile_vecs = (uint32_t)tile_vecs;
    p.seg_vecs = (uint32_t)((tile_vecs + segs - 1) / segs);
    p.row_vecs = (uint32_t)row_vecs;
    p.pix_vecs = (uint32_t)pix_vecs;
    p.div_row = make_fastdiv(p.row_vecs);
    p.div_segs = make_fastdiv((uint32_t)p.segs);
    hipStream_t s = (hipStream_t)stream;

#define SBNET_COPY_DT(MODE)                                                                              \
    (dt == SBNET_F32    ? dispatch_vec<MODE, SBNET_F32>(vec, img, tiles, indices, count, p, s)           \
     : dt == SBNET_BF16 ? dispatch_vec<MODE, SBNET_BF16>(vec, img, tiles, indices, count, p, s)          \
                        : dispatch_vec<MODE, SBNET_F16>(vec, img, tiles, indices, count, p, s))
    if (mode == 0) return SBNET_COPY_DT(0);
    if (mode == 1) return SBNET_COPY_DT(1);
    if (mode == 3) return SBNET_COPY_DT(3);
    return SBNET_COPY_DT(2);
#undef SBNET_COPY_DT
}

}  // namespace sbnet

using namespace sbnet;

extern "C" sbnet_status sbnet_sparse_gather(const void *x, sbnet_dtype dtype, int N, int H, int W, int C,
                                            const int32_t *indices, const int32_t *count, int cap,
                                            const sbnet_geom *g, void *tiles, void *stream) {
    return tile_copy_entry("sbnet_sparse_gather", 0, const_cast<void *>(x), tiles, dtype, N, H, W, C, indices,
                           count, cap, g, stream);
}

extern "C" sbnet_status sbnet_zero_outside(void *tiles, sbnet_dtype dtype, int H, int W, int C, const int32_t *indices,
                                           const int32_t *count, int cap, const sbnet_geom *g, void *stream) {
    // the image pointer is only checked for null and alignment in this mode: pass the tile stack
    return tile_copy_entry("sbnet_zero_outside", 3, tiles, tiles, dtype, 1, H, W, C, indices, count, cap, g, stream);
}

extern "C" sbnet_status sbnet_sparse_scatter(const void *tiles, sbnet_dtype dtype, const int32_t *indices,
                                             const int32_t *count, int cap, const sbnet_geom *g, void *y, int N,
                                             int H, int W, int C, int add, void *stream) {
    return tile_copy_entry("sbnet_sparse_scatter", add ? 2 : 1, y, const_cast<void *>(tiles), dtype, N, H, W, C,
                           indices, count, cap, g, stream);
}
