// The two small pieces that the backward pass of a chain of tile convolutions needs besides the convolutions' own
// gradients (training support for the residual unit of Sec. 3.3 of arXiv 1801.02108, composed from single calls):
//
//   tile_relu_backward   dout = dy where the forward activation y is positive, else 0, on the tiles
//                        b < min(*count, cap); tiles beyond the count are not touched.
//   tile_bias_partial +  db[c] = sum over those tiles and their pixels of dy[b][pixel][c]: workgroup w of G (at most 256)
//   tile_bias_sum        sums tiles w, w + G, ... per channel in fp32 (threads strided over pixels, one LDS reduction
//                        at the end), then one workgroup per 64 channels adds the G sums in a fixed order: no
//                        atomics, the same bits every run for a given cap.
//   both in one pass     tile_bias_partial<.., MASK> masks dy by y, writes it and sums what it wrote: the gradient
//                        that enters a convolution through its ReLU is read once for both.
#include "common.h"

namespace sbnet {
namespace {

template <int DT>
__device__ __forceinline__ float elem_to_float(uint32_t bits16or32) {
    if (DT == SBNET_F32) return __uint_as_float(bits16or32);
    if (DT == SBNET_BF16) return bf16_bits_to_float(bits16or32 & 0xffffu);
    union { _Float16 h[2]; uint32_t u; } v;
    v.u = bits16or32;
    return (float)v.h[0];
}

// words of 4 bytes: one f32 element or two 16-bit elements
template <int DT>
__device__ __forceinline__ uint32_t relu_mask_word(uint32_t y, uint32_t dy) {
    if (DT == SBNET_F32) return elem_to_float<DT>(y) > 0.f ? dy : 0u;
    const uint32_t lo = elem_to_float<DT>(y & 0xffffu) > 0.f ? 0xffffu : 0u;
    const uint32_t hi = elem_to_float<DT>(y >> 16) > 0.f ? 0xffff0000u : 0u;
    return dy & (lo | hi);
}

template <int DT>
__global__ __launch_bounds__(256) void tile_relu_backward(const uint32_t *__restrict__ y, const uint32_t *dy, uint32_t *dout,
                                                          const int32_t *__restrict__ count, int cap, size_t words_per_tile) {
    int n = *count;
    if (n > cap) n = cap;
    const size_t total = (size_t)(n > 0 ? n : 0) * words_per_tile;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    // four words per thread and step where the stack allows 16-byte accesses, single words for the tail
    const size_t vec_end = total & ~(size_t)3;
    for (; i < vec_end; i += stride * 4) {
        const uint4 a = *(const uint4 *)(y + i), g = *(const uint4 *)(dy + i);
        *(uint4 *)(dout + i) = make_uint4(relu_mask_word<DT>(a.x, g.x), relu_mask_word<DT>(a.y, g.y),
                                          relu_mask_word<DT>(a.z, g.z), relu_mask_word<DT>(a.w, g.w));
    }
    if (blockIdx.x == 0 && threadIdx.x < (unsigned)(total - vec_end))
        dout[vec_end + threadIdx.x] = relu_mask_word<DT>(y[vec_end + threadIdx.x], dy[vec_end + threadIdx.x]);
}

// part[w][c] = sum over the pixels of the tiles w, w + G, ... of workgroup w (G = gridDim.x).  VW = 4: a thread owns
// 16 bytes (4 words) of a pixel's channels and every (256 / vectors per pixel)-th pixel; VW = 1:
// one word, for channel counts that do not fill 16-byte vectors.  cw = 4-byte words per pixel (one f32 channel or two
// 16-bit ones), cw / VW <= 256.  Every thread adds its pixels tile after tile in ascending order; the pixel groups
// are then added in ascending order through LDS.
// MASK: the words of dy are first masked by the forward activation y (relu_mask_word), written to dout at the same
// place (dout may be dy: every word is read and written by one thread) and summed as written.
template <int DT, int VW, bool MASK>
__global__ __launch_bounds__(256) void tile_bias_partial(const uint32_t *dy, const int32_t *__restrict__ count,
                                                         int cap, int pixels, int C, int cw, float *__restrict__ part,
                                                         const uint32_t *__restrict__ y, uint32_t *dout) {
    constexpr int EPW = DT == SBNET_F32 ? 1 : 2;
    constexpr int NE = VW * EPW;                                  // channels per thread
    __shared__ float red[256][NE + 1];
    int n = *count;
    if (n > cap) n = cap;
    if ((int)blockIdx.x >= n) return;                             // the sum reads no result of this workgroup
    const int cvn = cw / VW;                                      // threads per pixel
    const int groups = 256 / cvn;                                 // pixel groups that fit the workgroup
    const int w = threadIdx.x % cvn, pg = threadIdx.x / cvn;
    float acc[NE];
#pragma unroll
    for (int e = 0; e < NE; ++e) acc[e] = 0.f;
    auto add = [&](const uint32_t *v) {
#pragma unroll
        for (int k = 0; k < VW; ++k) {
            if (DT == SBNET_F32) {
                acc[k] += __uint_as_float(v[k]);
            } else {
                acc[2 * k] += elem_to_float<DT>(v[k] & 0xffffu);
                acc[2 * k + 1] += elem_to_float<DT>(v[k] >> 16);
            }
        }
    };
    auto load = [](uint32_t *v, const uint32_t *q) {
        if (VW == 4) {
            const uint4 t = *(const uint4 *)q;
            v[0] = t.x; v[VW > 1 ? 1 : 0] = t.y; v[VW > 2 ? 2 : 0] = t.z; v[VW > 3 ? 3 : 0] = t.w;
        } else {
            v[0] = q[0];
        }
    };
    auto mask_store = [](uint32_t *v, const uint32_t *a, uint32_t *q) {
#pragma unroll
        for (int k = 0; k < VW; ++k) v[k] = relu_mask_word<DT>(a[k], v[k]);
        if (VW == 4) *(uint4 *)q = make_uint4(v[0], v[VW > 1 ? 1 : 0], v[VW > 2 ? 2 : 0], v[VW > 3 ? 3 : 0]);
        else q[0] = v[0];
    };
    if (pg < groups) {
        // the thread's pixels, tile after tile and in ascending order inside a tile, taken eight at a time whatever
        // the tile they fall in: eight (with a mask sixteen) loads are in flight all the way
        constexpr int U = 8;
        const int ppt = (pixels + groups - 1) / groups;           // pixel slots of this thread per tile
        const int total = ((n - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x) * ppt;
        int b = blockIdx.x, px = pg;                               // slot j: tile b, pixel px
        const size_t first = (size_t)blockIdx.x * pixels * cw + (size_t)w * VW;      // pixel 0 of the workgroup's first tile
        for (int j0 = 0; j0 < total; j0 += U) {
            uint32_t v[U][VW], a[U][VW];
            size_t off[U];
            bool ok[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                // a slot that holds no pixel reads pixel 0 of the first tile (always there) and is not used: no branch
                // between the loads
                ok[u] = j0 + u < total && px < pixels;
                off[u] = ok[u] ? ((size_t)b * pixels + px) * cw + (size_t)w * VW : first;
                load(v[u], dy + off[u]);
                if (MASK) load(a[u], y + off[u]);
                px += groups;
                if (px >= ppt * groups + pg) { px = pg; b += gridDim.x; }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (ok[u]) {
                    if (MASK) mask_store(v[u], a[u], dout + off[u]);
                    add(v[u]);
                }
            }
        }
    }
#pragma unroll
    for (int e = 0; e < NE; ++e) red[threadIdx.x][e] = acc[e];
    __syncthreads();
    if (threadIdx.x < (unsigned)cvn) {                            // groups in ascending order
        float a[NE];
#pragma unroll
        for (int e = 0; e < NE; ++e) a[e] = 0.f;
        for (int k = 0; k < groups; ++k)
#pragma unroll
            for (int e = 0; e < NE; ++e) a[e] += red[k * cvn + threadIdx.x][e];
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            const int c = threadIdx.x * NE + e;
            if (c < C) part[(size_t)blockIdx.x * C + c] = a[e];
        }
    }
}

// db[c] = sum over the workgroups' results part[w][c], w < min(n, G): 64 channels per workgroup of 16 waves; wave k takes
// the results k, k + 16, ... in ascending order, eight loads in flight, then the 16 sums are added in ascending order
__global__ __launch_bounds__(1024) void tile_bias_sum(const float *__restrict__ part, const int32_t *__restrict__ count, int cap,
                                                      int G, int C, float *__restrict__ db) {
    __shared__ float slice[16][64];
    const int lane = threadIdx.x & 63, k = threadIdx.x >> 6;
    const int c = blockIdx.x * 64 + lane;
    int n = *count;
    if (n > cap) n = cap;
    if (n > G) n = G;
    float acc = 0.f;
    if (c < C) {
        for (int b = k; b < n; b += 128) {
            float a[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int bj = b + 16 * j;
                const float v = part[(size_t)(bj < n ? bj : 0) * C + c];
                a[j] = bj < n ? v : 0.f;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) acc += a[j];
        }
    }
    slice[k][lane] = acc;
    __syncthreads();
    if (k == 0 && c < C) {
        float t = slice[0][lane];
#pragma unroll
        for (int i = 1; i < 16; ++i) t += slice[i][lane];
        db[c] = t;
    }
}

}  // namespace
}  // namespace sbnet

using namespace sbnet;

extern "C" sbnet_status sbnet_relu_backward_on_tiles(const void *y_tiles, const void *dy_tiles, sbnet_dtype dtype,
                                                     const int32_t *count, int cap, size_t tile_elems, void *dout_tiles,
                                                     void *stream) {
    const char *who = "sbnet_relu_backward_on_tiles";
    if (!y_tiles || !dy_tiles || !dout_tiles || !count) return fail(SBNET_EINVAL, "%s: null pointer", who);
    if (!is_float_dtype(dtype)) return fail(SBNET_EUNSUPPORTED, "%s: dtype must be f32, bf16 or f16", who);
    if (cap < 0 || tile_elems == 0) return fail(SBNET_EINVAL, "%s: bad sizes", who);
    if (((uintptr_t)y_tiles | (uintptr_t)dy_tiles | (uintptr_t)dout_tiles) & 15)
        return fail(SBNET_EINVAL, "%s: pointers must be 16-byte aligned", who);
    const size_t tile_bytes = tile_elems * elem_bytes(dtype);
    if (tile_bytes % 4) return fail(SBNET_EUNSUPPORTED, "%s: a tile must be a whole number of 4-byte words", who);
    if (cap == 0) return SBNET_OK;
    const size_t words = tile_bytes / 4;
    const size_t total = (size_t)cap * words;
    const size_t want = (total / 4 + 255) / 256;
    const int grid = (int)(want < 1 ? 1 : want > 2048 ? 2048 : want);
    hipStream_t s = (hipStream_t)stream;
#define SBNET_RB(DT) hipLaunchKernelGGL(tile_relu_backward<DT>, dim3(grid), dim3(256), 0, s, (const uint32_t *)y_tiles, \
                                        (const uint32_t *)dy_tiles, (uint32_t *)dout_tiles, count, cap, words)
    if (dtype == SBNET_F32) SBNET_RB(SBNET_F32);
    else if (dtype == SBNET_BF16) SBNET_RB(SBNET_BF16);
    else SBNET_RB(SBNET_F16);
#undef SBNET_RB
    return launch_status(who);
}

extern "C" size_t sbnet_bias_backward_workspace_bytes(int cap, int C) {
    if (cap < 0 || C <= 0) return 0;
    return ((size_t)(cap > 0 ? cap : 1) * C) * sizeof(float);
}

namespace {

// db = per-channel sum over the active tiles of dy (y == nullptr) or of dy masked by y > 0, which is also written to dout
sbnet_status bias_backward(const char *who, const void *y_tiles, const void *dy_tiles, sbnet_dtype dtype, const int32_t *count,
                           int cap, int pixels, int C, void *dout_tiles, float *db, void *workspace, size_t workspace_bytes,
                           void *stream) {
    const bool mask = y_tiles != nullptr;
    if (!dy_tiles || !count || !db || !workspace || (mask && !dout_tiles)) return fail(SBNET_EINVAL, "%s: null pointer", who);
    if (!is_float_dtype(dtype)) return fail(SBNET_EUNSUPPORTED, "%s: dtype must be f32, bf16 or f16", who);
    if (cap < 0 || pixels <= 0 || C <= 0) return fail(SBNET_EINVAL, "%s: bad sizes", who);
    const int es = elem_bytes(dtype);
    if ((long long)C * es % 4) return fail(SBNET_EUNSUPPORTED, "%s: a pixel's channels must fill 4-byte words", who);
    const int cw = C * es / 4;
    const uintptr_t ptrs = (uintptr_t)dy_tiles | (uintptr_t)y_tiles | (uintptr_t)(mask ? dout_tiles : nullptr);
    const bool vec = cw % 4 == 0 && (ptrs & 15) == 0;              // 16-byte accesses
    if ((vec ? cw / 4 : cw) > 256) return fail(SBNET_EUNSUPPORTED, "%s: too many channels per pixel", who);
    if ((ptrs & 3) || ((uintptr_t)workspace & 3)) return fail(SBNET_EINVAL, "%s: pointers must be 4-byte aligned", who);
    if (workspace_bytes < sbnet_bias_backward_workspace_bytes(cap, C)) return fail(SBNET_EINVAL, "%s: workspace too small", who);
    hipStream_t s = (hipStream_t)stream;
    float *part = (float *)workspace;
    if (cap > 0) {
        const int grid = cap < 256 ? cap : 256;
#define SBNET_BP2(DT, VW, MASK)                                                                                       \
    hipLaunchKernelGGL((tile_bias_partial<DT, VW, MASK>), dim3(grid), dim3(256), 0, s, (const uint32_t *)dy_tiles, count, \
                       cap, pixels, C, cw, part, (const uint32_t *)y_tiles, (uint32_t *)dout_tiles)
#define SBNET_BP(DT)                                                   \
    do {                                                              \
        if (vec && mask) SBNET_BP2(DT, 4, true);                      \
        else if (vec) SBNET_BP2(DT, 4, false);                        \
        else if (mask) SBNET_BP2(DT, 1, true);                        \
        else SBNET_BP2(DT, 1, false);                                 \
    } while (0)
        if (dtype == SBNET_F32) SBNET_BP(SBNET_F32);
        else if (dtype == SBNET_BF16) SBNET_BP(SBNET_BF16);
        else SBNET_BP(SBNET_F16);
#undef SBNET_BP
#undef SBNET_BP2
        sbnet_status st = launch_status(who);
        if (st != SBNET_OK) return st;
    }
    hipLaunchKernelGGL(tile_bias_sum, dim3((C + 63) / 64), dim3(1024), 0, s, part, count, cap, cap < 256 ? cap : 256, C, db);
    return launch_status(who);
}

}  // namespace

extern "C" sbnet_status sbnet_bias_backward_on_tiles(const void *dy_tiles, sbnet_dtype dtype, const int32_t *count, int cap,
                                                     int pixels, int C, float *db, void *workspace, size_t workspace_bytes,
                                                     void *stream) {
    return bias_backward("sbnet_bias_backward_on_tiles", nullptr, dy_tiles, dtype, count, cap, pixels, C, nullptr, db, workspace,
                         workspace_bytes, stream);
}

extern "C" sbnet_status sbnet_relu_bias_backward_on_tiles(const void *y_tiles, const void *dy_tiles, sbnet_dtype dtype,
                                                          const int32_t *count, int cap, int pixels, int C, void *dout_tiles,
                                                          float *db, void *workspace, size_t workspace_bytes, void *stream) {
    if (!y_tiles) return fail(SBNET_EINVAL, "sbnet_relu_bias_backward_on_tiles: null pointer");
    return bias_backward("sbnet_relu_bias_backward_on_tiles", y_tiles, dy_tiles, dtype, count, cap, pixels, C, dout_tiles, db,
                         workspace, workspace_bytes, stream);
}
