// Gradient of the overlapping gather (end of Sec. 3.3 of arXiv 1801.02108, "End-to-end training of SBNet"): the
// gradient of a gather is a scatter-add of the tile gradients, and because neighbouring tiles share their halo, a
// pixel on a tile edge receives contributions from up to four tiles.  (The gradient of the scatter is the plain
// gather and needs no kernel of its own.)
//
// The paper adds with atomics.  Here the sum is pulled instead of pushed: a small map from block coordinates to
// the block's position in the index list is built first (two tiny kernels), then every cell of the block grid
// (bstride_h x bstride_w pixels) looks up the at most (R+1)^2 tiles that can cover it, R = ceil((bsize - bstride) /
// bstride), and each of its pixels adds their contributions in ascending (by, bx) order, in fp32, onto dx, rounding
// once.  No atomics, results do not depend on scheduling, every dx vector is read and written once, whole vectors.
#include "tile_add.h"

namespace sbnet {

constexpr int kGbThreads = 256;
constexpr int kGbMaxR = 3;       // tiles may reach over at most three following cells per axis

struct GbParams {
    sbnet_geom g;
    int N, H, W, cap;
    int cells_h, cells_w;        // cells that a tile can touch: bcount + R
    int R_h, R_w;
    uint32_t pix_vecs;           // vectors per pixel
    uint32_t cell_vecs;          // vectors per cell: bstride_h * bstride_w * pix_vecs
    uint32_t row_vecs;           // vectors per cell row: bstride_w * pix_vecs
    uint32_t tile_row_vecs;      // vectors per tile row: bsize_w * pix_vecs
    uint32_t tile_vecs;
    FastDiv div_cells, div_cw, div_row, div_pv;
};

__global__ void gb_map_clear(int32_t *map, int n) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) map[i] = -1;
}

__global__ void gb_map_fill(int32_t *map, const int32_t *__restrict__ indices, const int32_t *__restrict__ count,
                            int cap, int N, int bh, int bw) {
    const int nact = min(*count, cap);
    for (int b = blockIdx.x * blockDim.x + threadIdx.x; b < nact; b += gridDim.x * blockDim.x) {
        const int n = indices[3 * b], by = indices[3 * b + 1], bx = indices[3 * b + 2];
        if (n >= 0 && n < N && by >= 0 && by < bh && bx >= 0 && bx < bw) map[(n * bh + by) * bw + bx] = b;
    }
}

// both steps in one workgroup (one launch less) when the map and the list are small enough for it
__global__ __launch_bounds__(1024) void gb_map_build(int32_t *map, int nmap, const int32_t *__restrict__ indices,
                                                     const int32_t *__restrict__ count, int cap, int N, int bh, int bw) {
    for (int i = threadIdx.x; i < nmap; i += blockDim.x) map[i] = -1;
    __syncthreads();
    const int nact = min(*count, cap);
    for (int b = threadIdx.x; b < nact; b += blockDim.x) {
        const int n = indices[3 * b], by = indices[3 * b + 1], bx = indices[3 * b + 2];
        if (n >= 0 && n < N && by >= 0 && by < bh && bx >= 0 && bx < bw) map[(n * bh + by) * bw + bx] = b;
    }
}

// fp32 sum of storage words, element-wise
template <int DT> struct Acc;
template <> struct Acc<SBNET_F32> {
    static constexpr int N = 1;
    static __device__ __forceinline__ void add(float *a, uint32_t w) { a[0] += __uint_as_float(w); }
    static __device__ __forceinline__ uint32_t pack(const float *a) { return __float_as_uint(a[0]); }
};
template <> struct Acc<SBNET_BF16> {
    static constexpr int N = 2;
    static __device__ __forceinline__ void add(float *a, uint32_t w) {
        a[0] += bf16_bits_to_float(w & 0xffffu);
        a[1] += bf16_bits_to_float(w >> 16);
    }
    static __device__ __forceinline__ uint32_t pack(const float *a) {
        return float_to_bf16_bits(a[0]) | (float_to_bf16_bits(a[1]) << 16);
    }
};
template <> struct Acc<SBNET_F16> {
    static constexpr int N = 2;
    static __device__ __forceinline__ float h2f(uint32_t b) {
        union { _Float16 h; uint16_t u; } x;
        x.u = (uint16_t)b;
        return (float)x.h;
    }
    static __device__ __forceinline__ uint32_t f2h(float f) {
        union { _Float16 h; uint16_t u; } x;
        x.h = (_Float16)f;
        return x.u;
    }
    static __device__ __forceinline__ void add(float *a, uint32_t w) {
        a[0] += h2f(w & 0xffffu);
        a[1] += h2f(w >> 16);
    }
    static __device__ __forceinline__ uint32_t pack(const float *a) { return f2h(a[0]) | (f2h(a[1]) << 16); }
};

// V: uint4 / uint2 / uint32_t (whole 32-bit words of the storage type)
template <typename V> struct Words;
template <> struct Words<uint4> { static constexpr int N = 4; };
template <> struct Words<uint2> { static constexpr int N = 2; };
template <> struct Words<uint32_t> { static constexpr int N = 1; };
__device__ __forceinline__ uint32_t word_of(const uint4 &v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }
__device__ __forceinline__ uint32_t word_of(const uint2 &v, int i) { return i == 0 ? v.x : v.y; }
__device__ __forceinline__ uint32_t word_of(const uint32_t &v, int) { return v; }
__device__ __forceinline__ void make_vec(uint4 &v, const uint32_t *w) { v = make_uint4(w[0], w[1], w[2], w[3]); }
__device__ __forceinline__ void make_vec(uint2 &v, const uint32_t *w) { v = make_uint2(w[0], w[1]); }
__device__ __forceinline__ void make_vec(uint32_t &v, const uint32_t *w) { v = w[0]; }

// RM: largest reach (in cells) this instantiation handles; U vectors per thread are processed together, all of
// their loads (tile gradients and dx) issued before the first is used: a thread's memory round trips overlap
// instead of adding up (more than two at a time was measured slower: fewer workgroups fit a CU).
template <typename V, int DT, int RM, int U>
__global__ __launch_bounds__(kGbThreads) void gb_accumulate(V *__restrict__ dx, const V *__restrict__ dtiles,
                                                            const int32_t *__restrict__ map, GbParams p) {
    constexpr int NW = Words<V>::N, NA = Acc<DT>::N;
    constexpr int NT = (RM + 1) * (RM + 1);
    const uint32_t ncells = (uint32_t)p.N * p.cells_h * p.cells_w;
    for (uint32_t cell = blockIdx.x; cell < ncells; cell += gridDim.x) {
        const uint32_t n = fdiv(cell, p.div_cells);
        const uint32_t rest = cell - n * (uint32_t)(p.cells_h * p.cells_w);
        const int cy = (int)fdiv(rest, p.div_cw), cx = (int)rest - cy * p.cells_w;
        // tiles that can cover this cell: blocks (cy - R_h .. cy, cx - R_w .. cx), ascending; the lookups are
        // issued together (indices clamped into the map, results masked)
        int tb[NT];
        int nt = 0;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int dy = RM - t / (RM + 1), dxc = RM - t % (RM + 1);
            const int by = cy - dy, bx = cx - dxc;
            const bool ok = dy <= p.R_h && dxc <= p.R_w && by >= 0 && by < p.g.bcount_h && bx >= 0 && bx < p.g.bcount_w;
            const int e = map[((int)n * p.g.bcount_h + min(max(by, 0), p.g.bcount_h - 1)) * p.g.bcount_w +
                              min(max(bx, 0), p.g.bcount_w - 1)];
            tb[t] = ok ? e : -1;
            nt += tb[t] >= 0;
        }
        if (nt == 0) continue;                                   // workgroup-uniform
        const int py0 = p.g.boffset_h + cy * p.g.bstride_h, px0 = p.g.boffset_w + cx * p.g.bstride_w;
        for (uint32_t v0 = threadIdx.x; v0 < p.cell_vecs; v0 += kGbThreads * U) {
            V tv[U][NT], old[U];
            bool use[U][NT], any[U];
            size_t o[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t v = v0 + u * kGbThreads;
                const uint32_t r = fdiv(v, p.div_row), rem = v - r * p.row_vecs;
                const uint32_t c = fdiv(rem, p.div_pv), k = rem - c * p.pix_vecs;
                const int yy = py0 + (int)r, xx = px0 + (int)c;
                const bool live = v < p.cell_vecs && yy >= 0 && yy < p.H && xx >= 0 && xx < p.W;
                any[u] = false;
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const int dy = RM - t / (RM + 1), dxc = RM - t % (RM + 1);
                    // position inside that tile: its origin lies dy (dxc) cells up (left)
                    const int i = (int)r + dy * p.g.bstride_h, j = (int)c + dxc * p.g.bstride_w;
                    use[u][t] = live && tb[t] >= 0 && i < p.g.bsize_h && j < p.g.bsize_w;
                    if (use[u][t])
                        tv[u][t] = dtiles[(size_t)tb[t] * p.tile_vecs + (uint32_t)i * p.tile_row_vecs + (uint32_t)j * p.pix_vecs + k];
                    any[u] |= use[u][t];
                }
                o[u] = (((size_t)n * p.H + yy) * p.W + xx) * p.pix_vecs + k;
                if (any[u]) old[u] = dx[o[u]];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (!any[u]) continue;
                float acc[NW * NA];
#pragma unroll
                for (int i = 0; i < NW * NA; ++i) acc[i] = 0.f;
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    if (use[u][t]) {
#pragma unroll
                        for (int w = 0; w < NW; ++w) Acc<DT>::add(acc + w * NA, word_of(tv[u][t], w));
                    }
                uint32_t out[NW];
#pragma unroll
                for (int w = 0; w < NW; ++w) {
                    Acc<DT>::add(acc + w * NA, word_of(old[u], w));
                    out[w] = Acc<DT>::pack(acc + w * NA);
                }
                V res;
                make_vec(res, out);
                dx[o[u]] = res;
            }
        }
    }
}

template <typename V, int DT>
static void launch_gb(void *dx, const void *dtiles, const int32_t *map, const GbParams &p, hipStream_t s) {
    const long long ncells = (long long)p.N * p.cells_h * p.cells_w;
    const int grid = (int)(ncells < 16384 ? ncells : 16384);
    if (p.R_h <= 1 && p.R_w <= 1)
        hipLaunchKernelGGL((gb_accumulate<V, DT, 1, 2>), dim3(grid), dim3(kGbThreads), 0, s, (V *)dx, (const V *)dtiles, map, p);
    else
        hipLaunchKernelGGL((gb_accumulate<V, DT, kGbMaxR, 2>), dim3(grid), dim3(kGbThreads), 0, s, (V *)dx, (const V *)dtiles, map, p);
}

template <int DT>
static sbnet_status dispatch_gb(int vec_bytes, void *dx, const void *dtiles, const int32_t *map, const GbParams &p,
                                hipStream_t s) {
    switch (vec_bytes) {
        case 16: launch_gb<uint4, DT>(dx, dtiles, map, p, s); break;
        case 8: launch_gb<uint2, DT>(dx, dtiles, map, p, s); break;
        case 4: launch_gb<uint32_t, DT>(dx, dtiles, map, p, s); break;
        default: return fail(SBNET_EUNSUPPORTED, "sbnet_sparse_gather_backward: a pixel's channels must fill 4-byte words");
    }
    return launch_status("sbnet_sparse_gather_backward");
}

}  // namespace sbnet

using namespace sbnet;

extern "C" size_t sbnet_gather_backward_workspace_bytes(int N, const sbnet_geom *g) {
    if (N <= 0 || !geom_ok(g)) return 0;
    return (size_t)N * g->bcount_h * g->bcount_w * sizeof(int32_t);
}

extern "C" sbnet_status sbnet_sparse_gather_backward(const void *dtiles, sbnet_dtype dtype, const int32_t *indices,
                                                     const int32_t *count, int cap, const sbnet_geom *g, void *dx,
                                                     int N, int H, int W, int C, void *workspace,
                                                     size_t workspace_bytes, void *stream) {
    const char *who = "sbnet_sparse_gather_backward";
    if (!dtiles || !indices || !count || !dx || !workspace) return fail(SBNET_EINVAL, "%s: null pointer", who);
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || cap < 0) return fail(SBNET_EINVAL, "%s: bad sizes", who);
    if (!geom_ok(g)) return fail(SBNET_EINVAL, "%s: bad geometry", who);
    if (!is_float_dtype(dtype)) return fail(SBNET_EUNSUPPORTED, "%s: dtype must be f32, bf16 or f16", who);
    if (((uintptr_t)dx | (uintptr_t)dtiles) & 15 || ((uintptr_t)workspace & 3))
        return fail(SBNET_EINVAL, "%s: pointers must be 16-byte aligned (workspace: 4)", who);
    if (workspace_bytes < sbnet_gather_backward_workspace_bytes(N, g)) return fail(SBNET_EINVAL, "%s: workspace too small", who);
    const int R_h = g->bsize_h > g->bstride_h ? (g->bsize_h - g->bstride_h + g->bstride_h - 1) / g->bstride_h : 0;
    const int R_w = g->bsize_w > g->bstride_w ? (g->bsize_w - g->bstride_w + g->bstride_w - 1) / g->bstride_w : 0;
    if (R_h > kGbMaxR || R_w > kGbMaxR)
        return fail(SBNET_EUNSUPPORTED, "%s: tiles may overlap at most three following blocks per axis", who);
    if (cap == 0) return SBNET_OK;
    const long long pix_bytes = (long long)C * elem_bytes(dtype);
    int vec = 16;
    while (vec > 4 && pix_bytes % vec) vec >>= 1;
    if (pix_bytes % vec) return fail(SBNET_EUNSUPPORTED, "%s: a pixel's channels must fill 4-byte words", who);
    const long long cells = (long long)N * (g->bcount_h + R_h) * (g->bcount_w + R_w);
    const long long tile_vecs = (long long)g->bsize_h * g->bsize_w * (pix_bytes / vec);
    if (cells >= (1LL << 31) || tile_vecs >= (1LL << 31) || (long long)N * g->bcount_h * g->bcount_w >= (1LL << 31) ||
        (long long)g->bstride_h * g->bstride_w * (pix_bytes / vec) >= (1LL << 31))
        return fail(SBNET_EUNSUPPORTED, "%s: tensor too large", who);

    GbParams p;
    p.g = *g;
    p.N = N; p.H = H; p.W = W; p.cap = cap;
    p.R_h = R_h; p.R_w = R_w;
    p.cells_h = g->bcount_h + R_h;
    p.cells_w = g->bcount_w + R_w;
    p.pix_vecs = (uint32_t)(pix_bytes / vec);
    p.row_vecs = (uint32_t)g->bstride_w * p.pix_vecs;
    p.cell_vecs = (uint32_t)g->bstride_h * p.row_vecs;
    p.tile_row_vecs = (uint32_t)g->bsize_w * p.pix_vecs;
    p.tile_vecs = (uint32_t)tile_vecs;
    p.div_cells = make_fastdiv((uint32_t)(p.cells_h * p.cells_w));
    p.div_cw = make_fastdiv((uint32_t)p.cells_w);
    p.div_row = make_fastdiv(p.row_vecs);
    p.div_pv = make_fastdiv(p.pix_vecs);
    hipStream_t s = (hipStream_t)stream;
    int32_t *map = (int32_t *)workspace;
    const int nmap = N * g->bcount_h * g->bcount_w;
    if (nmap <= 32768 && cap <= 32768) {
        hipLaunchKernelGGL(gb_map_build, dim3(1), dim3(1024), 0, s, map, nmap, indices, count, cap, N, g->bcount_h, g->bcount_w);
    } else {
        hipLaunchKernelGGL(gb_map_clear, dim3((nmap + 255) / 256 > 1024 ? 1024 : (nmap + 255) / 256), dim3(256), 0, s, map, nmap);
        hipLaunchKernelGGL(gb_map_fill, dim3((cap + 255) / 256 > 1024 ? 1024 : (cap + 255) / 256), dim3(256), 0, s, map, indices,
                           count, cap, N, g->bcount_h, g->bcount_w);
    }
    if (dtype == SBNET_F32) return dispatch_gb<SBNET_F32>(vec, dx, dtiles, map, p, s);
    if (dtype == SBNET_BF16) return dispatch_gb<SBNET_BF16>(vec, dx, dtiles, map, p, s);
    return dispatch_gb<SBNET_F16>(vec, dx, dtiles, map, p, s);
}
