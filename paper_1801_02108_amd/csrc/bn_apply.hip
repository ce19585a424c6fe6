// Batch normalisation over the active blocks only (Sec. 3.3 of arXiv 1801.02108: the layers of a residual unit run in
// sparse mode and normalise across the non-sparse elements), forward and backward, on the feature map in place of
// the tile stack: non-overlapping blocks, every active pixel once.
//
//   bn_apply        y = act(gamma (x - mean) / sqrt(var + eps) + beta) on the pixels of the listed blocks that lie
//                   inside the image; every other pixel of y is left as it is.
//   bn_bwd_partial  with z = gamma xhat + beta, g = dy (or dy where z > 0 when the forward call applied a ReLU):
//                   per (block, channel) the sums of g and of g xhat, reduced through LDS.
//   bn_bwd_combine  per channel: dbeta = sum g, dgamma = sum g xhat over the blocks (every thread a strided subset in
//                   list order, then a fixed tree: no atomics, the same bits every run), and the pixel count.
//   bn_bwd_dx       dx = gamma / sqrt(var + eps) * (g - dbeta / n - xhat dgamma / n): the gradient of training-mode
//                   normalisation whose mean and variance are the statistics of these same n pixels.
//
// All four walk (block, slab of 128 bytes of channels per pixel) items with 8 lanes per pixel strip, as the statistics
// kernel does; arithmetic in fp32, one rounding to the storage type.
#include "bn_common.h"

namespace sbnet {
namespace {

struct BnAffine {
    const float *mean, *var, *gamma, *beta;   // gamma, beta may be null (1, 0)
    float eps;
    int relu;
};

// origin of block b's window and this thread's place in the slab
struct BnPlace {
    int y0, x0, npx, c0;
    bool chan_ok;
    long long base;
};

template <int EPV>
__device__ __forceinline__ BnPlace bn_place(uint32_t b, int slab, int k, const int32_t *indices, const BnParams &p) {
    BnPlace w;
    const int n = indices[3 * b], by = indices[3 * b + 1], bx = indices[3 * b + 2];
    w.y0 = p.g.boffset_h + by * p.g.bstride_h;
    w.x0 = p.g.boffset_w + bx * p.g.bstride_w;
    const int ylo = max(w.y0, 0), yhi = min(w.y0 + p.g.bsize_h, p.H), xlo = max(w.x0, 0), xhi = min(w.x0 + p.g.bsize_w, p.W);
    w.npx = max(yhi - ylo, 0) * max(xhi - xlo, 0);
    w.c0 = slab * p.cs + k * EPV;
    w.chan_ok = w.c0 < p.C;
    w.base = (long long)n * p.H * p.W * p.pix_vecs + (long long)(slab * (p.cs / EPV) + k);
    return w;
}

// vector index of pixel q of the block (row-major inside the window), or -1 outside the image / the block
__device__ __forceinline__ long long bn_pixel(const BnPlace &w, int q, const BnParams &p) {
    const int i = (int)fdiv((uint32_t)q, p.div_w), j = q - i * p.g.bsize_w;
    const int yy = w.y0 + i, xx = w.x0 + j;
    if (!w.chan_ok || q >= p.hw || yy < 0 || yy >= p.H || xx < 0 || xx >= p.W) return -1;
    return w.base + ((long long)yy * p.W + xx) * p.pix_vecs;
}

template <int EPV>
__device__ __forceinline__ void bn_coeffs(const BnAffine &a, const BnPlace &w, int C, float *mean, float *rstd, float *gam,
                                          float *bet) {
#pragma unroll
    for (int e = 0; e < EPV; ++e) {
        const int c = w.c0 + e;
        const bool ok = w.chan_ok && c < C;
        mean[e] = ok ? a.mean[c] : 0.f;
        rstd[e] = ok ? 1.0f / sqrtf(a.var[c] + a.eps) : 0.f;
        gam[e] = ok ? (a.gamma ? a.gamma[c] : 1.f) : 0.f;
        bet[e] = ok ? (a.beta ? a.beta[c] : 0.f) : 0.f;
    }
}

template <int DT>
__global__ __launch_bounds__(kBnThreads) void bn_apply(const uint4 *x, uint4 *y,                       // y may be x
                                                       const int32_t *__restrict__ indices, const int32_t *__restrict__ count,
                                                       BnParams p, BnAffine a) {
    constexpr int EPV = BnElem<DT>::EPV;
    const int nact = min(*count, p.cap);
    const uint32_t items = (uint32_t)nact * (uint32_t)p.slabs;
    const int pg = threadIdx.x >> 3, k = threadIdx.x & 7;
    for (uint32_t item = blockIdx.x; item < items; item += gridDim.x) {
        const uint32_t b = fdiv(item, p.div_slabs);
        const BnPlace w = bn_place<EPV>(b, (int)(item - b * p.slabs), k, indices, p);
        float mean[EPV], rstd[EPV], gam[EPV], bet[EPV];
        bn_coeffs<EPV>(a, w, p.C, mean, rstd, gam, bet);
        for (int q0 = pg; q0 < p.hw; q0 += 32 * 4) {
            long long at[4];
            uint4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                at[u] = bn_pixel(w, q0 + 32 * u, p);
                v[u] = make_uint4(0, 0, 0, 0);
                if (at[u] >= 0) v[u] = x[at[u]];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (at[u] >= 0) {
                    float f[EPV];
                    BnElem<DT>::unpack(v[u], f);
#pragma unroll
                    for (int e = 0; e < EPV; ++e) {
                        const float z = fmaf(gam[e], (f[e] - mean[e]) * rstd[e], bet[e]);
                        f[e] = a.relu ? fmaxf(z, 0.f) : z;
                    }
                    // a vector that straddles the channel count cannot occur: a pixel's channels fill whole vectors
                    y[at[u]] = bn_pack<DT>(f);
                }
        }
    }
}

// workspace layout: float part[cap][C][2] (sum g, sum g xhat), float cnt[cap], float ntot
template <int DT>
__global__ __launch_bounds__(kBnThreads) void bn_bwd_partial(const uint4 *__restrict__ x, const uint4 *__restrict__ dy,
                                                             const int32_t *__restrict__ indices,
                                                             const int32_t *__restrict__ count, float *__restrict__ part,
                                                             float *__restrict__ cnt, BnParams p, BnAffine a) {
    constexpr int EPV = BnElem<DT>::EPV;
    __shared__ float red[2][32][8 * EPV + 1];
    const int nact = min(*count, p.cap);
    const uint32_t items = (uint32_t)nact * (uint32_t)p.slabs;
    const int pg = threadIdx.x >> 3, k = threadIdx.x & 7;
    for (uint32_t item = blockIdx.x; item < items; item += gridDim.x) {
        const uint32_t b = fdiv(item, p.div_slabs);
        const int slab = (int)(item - b * p.slabs);
        const BnPlace w = bn_place<EPV>(b, slab, k, indices, p);
        float mean[EPV], rstd[EPV], gam[EPV], bet[EPV], s1[EPV], s2[EPV];
        bn_coeffs<EPV>(a, w, p.C, mean, rstd, gam, bet);
#pragma unroll
        for (int e = 0; e < EPV; ++e) s1[e] = s2[e] = 0.f;
        for (int q0 = pg; q0 < p.hw; q0 += 32 * 2) {
            long long at[2];
            uint4 vx[2], vg[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                at[u] = bn_pixel(w, q0 + 32 * u, p);
                vx[u] = vg[u] = make_uint4(0, 0, 0, 0);
                if (at[u] >= 0) {
                    vx[u] = x[at[u]];
                    vg[u] = dy[at[u]];
                }
            }
#pragma unroll
            for (int u = 0; u < 2; ++u)
                if (at[u] >= 0) {
                    float f[EPV], g[EPV];
                    BnElem<DT>::unpack(vx[u], f);
                    BnElem<DT>::unpack(vg[u], g);
#pragma unroll
                    for (int e = 0; e < EPV; ++e) {
                        const float xh = (f[e] - mean[e]) * rstd[e];
                        const float ge = (a.relu && !(fmaf(gam[e], xh, bet[e]) > 0.f)) ? 0.f : g[e];
                        s1[e] += ge;
                        s2[e] = fmaf(ge, xh, s2[e]);
                    }
                }
        }
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            red[0][pg][k * EPV + e] = s1[e];
            red[1][pg][k * EPV + e] = s2[e];
        }
        __syncthreads();
        if (threadIdx.x < 8 * EPV) {
            const int c = slab * p.cs + threadIdx.x;
            float t1 = 0.f, t2 = 0.f;
            for (int gq = 0; gq < 32; ++gq) {
                t1 += red[0][gq][threadIdx.x];
                t2 += red[1][gq][threadIdx.x];
            }
            if (c < p.C) {
                part[((size_t)b * p.C + c) * 2] = t1;
                part[((size_t)b * p.C + c) * 2 + 1] = t2;
            }
            if (slab == 0 && threadIdx.x == 0) cnt[b] = (float)w.npx;
        }
        __syncthreads();
    }
}

__global__ __launch_bounds__(kBnThreads) void bn_bwd_combine(const float *__restrict__ part, const float *__restrict__ cnt,
                                                             const int32_t *__restrict__ count, int cap, int C,
                                                             float *__restrict__ dgamma, float *__restrict__ dbeta,
                                                             float *__restrict__ ntot) {
    __shared__ float s1[kBnThreads], s2[kBnThreads], sn[kBnThreads];
    const int c = blockIdx.x;
    const int nact = min(*count, cap);
    float a = 0.f, q = 0.f, n = 0.f;
    for (int b = threadIdx.x; b < nact; b += kBnThreads) {
        a += part[((size_t)b * C + c) * 2];
        q += part[((size_t)b * C + c) * 2 + 1];
        n += cnt[b];
    }
    s1[threadIdx.x] = a; s2[threadIdx.x] = q; sn[threadIdx.x] = n;
    __syncthreads();
    for (int half = kBnThreads / 2; half > 0; half >>= 1) {
        if ((int)threadIdx.x < half) {
            s1[threadIdx.x] += s1[threadIdx.x + half];
            s2[threadIdx.x] += s2[threadIdx.x + half];
            sn[threadIdx.x] += sn[threadIdx.x + half];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        dbeta[c] = s1[0];
        dgamma[c] = s2[0];
        if (c == 0) *ntot = sn[0];
    }
}

template <int DT>
__global__ __launch_bounds__(kBnThreads) void bn_bwd_dx(const uint4 *__restrict__ x, const uint4 *dy,
                                                        uint4 *dx /* may be dy */, const int32_t *__restrict__ indices,
                                                        const int32_t *__restrict__ count, const float *__restrict__ dgamma,
                                                        const float *__restrict__ dbeta, const float *__restrict__ ntot,
                                                        BnParams p, BnAffine a) {
    constexpr int EPV = BnElem<DT>::EPV;
    const int nact = min(*count, p.cap);
    const uint32_t items = (uint32_t)nact * (uint32_t)p.slabs;
    const int pg = threadIdx.x >> 3, k = threadIdx.x & 7;
    const float n = *ntot, inv_n = n > 0.f ? 1.0f / n : 0.f;
    for (uint32_t item = blockIdx.x; item < items; item += gridDim.x) {
        const uint32_t b = fdiv(item, p.div_slabs);
        const BnPlace w = bn_place<EPV>(b, (int)(item - b * p.slabs), k, indices, p);
        float mean[EPV], rstd[EPV], gam[EPV], bet[EPV], mg[EPV], mgx[EPV];
        bn_coeffs<EPV>(a, w, p.C, mean, rstd, gam, bet);
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            const bool ok = w.chan_ok && w.c0 + e < p.C;
            mg[e] = ok ? dbeta[w.c0 + e] * inv_n : 0.f;
            mgx[e] = ok ? dgamma[w.c0 + e] * inv_n : 0.f;
        }
        for (int q0 = pg; q0 < p.hw; q0 += 32 * 2) {
            long long at[2];
            uint4 vx[2], vg[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                at[u] = bn_pixel(w, q0 + 32 * u, p);
                vx[u] = vg[u] = make_uint4(0, 0, 0, 0);
                if (at[u] >= 0) {
                    vx[u] = x[at[u]];
                    vg[u] = dy[at[u]];
                }
            }
#pragma unroll
            for (int u = 0; u < 2; ++u)
                if (at[u] >= 0) {
                    float f[EPV], g[EPV];
                    BnElem<DT>::unpack(vx[u], f);
                    BnElem<DT>::unpack(vg[u], g);
#pragma unroll
                    for (int e = 0; e < EPV; ++e) {
                        const float xh = (f[e] - mean[e]) * rstd[e];
                        const float ge = (a.relu && !(fmaf(gam[e], xh, bet[e]) > 0.f)) ? 0.f : g[e];
                        f[e] = gam[e] * rstd[e] * (ge - mg[e] - xh * mgx[e]);
                    }
                    dx[at[u]] = bn_pack<DT>(f);
                }
        }
    }
}

int bn_grid(int cap, const BnParams &p) {
    const long long items = (long long)cap * p.slabs;
    return (int)(items < 8192 ? items : 8192);
}

}  // namespace
}  // namespace sbnet

using namespace sbnet;

#define SBNET_BN_DISPATCH(KERNEL, ...)                                                                              \
    do {                                                                                                            \
        if (dtype == SBNET_F32) hipLaunchKernelGGL(KERNEL<SBNET_F32>, dim3(grid), dim3(kBnThreads), 0, s, __VA_ARGS__); \
        else if (dtype == SBNET_BF16) hipLaunchKernelGGL(KERNEL<SBNET_BF16>, dim3(grid), dim3(kBnThreads), 0, s, __VA_ARGS__); \
        else hipLaunchKernelGGL(KERNEL<SBNET_F16>, dim3(grid), dim3(kBnThreads), 0, s, __VA_ARGS__);                  \
    } while (0)

extern "C" sbnet_status sbnet_sparse_bn_apply(const void *x, sbnet_dtype dtype, int N, int H, int W, int C,
                                              const int32_t *indices, const int32_t *count, int cap, const sbnet_geom *g,
                                              const float *mean, const float *var, const float *gamma, const float *beta,
                                              float eps, int relu, void *y, void *stream) {
    const char *who = "sbnet_sparse_bn_apply";
    if (!x || !y || !indices || !count || !mean || !var) return fail(SBNET_EINVAL, "%s: null pointer", who);
    if (!(eps >= 0.f)) return fail(SBNET_EINVAL, "%s: eps must not be negative", who);
    BnParams p;
    sbnet_status st = bn_fill_params(who, dtype, N, H, W, C, cap, g, &p);
    if (st != SBNET_OK) return st;
    if (((uintptr_t)x | (uintptr_t)y) & 15) return fail(SBNET_EINVAL, "%s: x and y must be 16-byte aligned", who);
    if (cap == 0) return SBNET_OK;
    hipStream_t s = (hipStream_t)stream;
    const BnAffine a = {mean, var, gamma, beta, eps, relu ? 1 : 0};
    const int grid = bn_grid(cap, p);
    SBNET_BN_DISPATCH(bn_apply, (const uint4 *)x, (uint4 *)y, indices, count, p, a);
    return launch_status(who);
}

extern "C" size_t sbnet_bn_backward_workspace_bytes(int cap, int C) {
    if (cap < 0 || C <= 0) return 0;
    return ((size_t)cap * C * 2 + (size_t)cap + 1) * sizeof(float);
}

extern "C" sbnet_status sbnet_sparse_bn_backward(const void *x, const void *dy, sbnet_dtype dtype, int N, int H, int W, int C,
                                                 const int32_t *indices, const int32_t *count, int cap,
                                                 const sbnet_geom *g, const float *mean, const float *var,
                                                 const float *gamma, const float *beta, float eps, int relu, void *dx,
                                                 float *dgamma, float *dbeta, void *workspace, size_t workspace_bytes,
                                                 void *stream) {
    const char *who = "sbnet_sparse_bn_backward";
    if (!x || !dy || !dx || !indices || !count || !mean || !var || !dgamma || !dbeta)
        return fail(SBNET_EINVAL, "%s: null pointer", who);
    if (!(eps >= 0.f)) return fail(SBNET_EINVAL, "%s: eps must not be negative", who);
    BnParams p;
    sbnet_status st = bn_fill_params(who, dtype, N, H, W, C, cap, g, &p);
    if (st != SBNET_OK) return st;
    if (((uintptr_t)x | (uintptr_t)dy | (uintptr_t)dx) & 15)
        return fail(SBNET_EINVAL, "%s: x, dy and dx must be 16-byte aligned", who);
    if (!workspace || ((uintptr_t)workspace & 3) || workspace_bytes < sbnet_bn_backward_workspace_bytes(cap, C))
        return fail(SBNET_EINVAL, "%s: workspace missing, misaligned or too small", who);
    hipStream_t s = (hipStream_t)stream;
    const BnAffine a = {mean, var, gamma, beta, eps, relu ? 1 : 0};
    float *part = (float *)workspace;
    float *cnt = part + (size_t)cap * C * 2;
    float *ntot = cnt + cap;
    const int grid = cap > 0 ? bn_grid(cap, p) : 0;
    if (cap > 0) SBNET_BN_DISPATCH(bn_bwd_partial, (const uint4 *)x, (const uint4 *)dy, indices, count, part, cnt, p, a);
    hipLaunchKernelGGL(bn_bwd_combine, dim3(C), dim3(kBnThreads), 0, s, part, cnt, count, cap, C, dgamma, dbeta, ntot);
    if (cap > 0) SBNET_BN_DISPATCH(bn_bwd_dx, (const uint4 *)x, (const uint4 *)dy, (uint4 *)dx, indices, count, dgamma, dbeta, ntot, p, a);
    return launch_status(who);
}
