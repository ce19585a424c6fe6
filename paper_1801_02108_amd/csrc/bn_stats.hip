// Batch-norm statistics over the active blocks only (Sec. 3.3 of arXiv 1801.02108: the layers of a residual unit
// run in sparse mode, and normalising across the non-sparse elements alone keeps invalid data out of the
// statistics): per channel, the mean and the (biased) variance of x over the pixels of the listed blocks that lie
// inside the image.
//
// Two kernels, no atomics, fixed summation order:
//   bn_partial   one workgroup per (active block, slab of 128 bytes of channels per pixel).  Eight lanes read one
//                pixel's 128-byte strip; a thread accumulates, in fp32, the sum and the sum of squares of its
//                channels over every 32nd pixel, taken relative to the block's first pixel (which keeps the squares
//                small when the mean is large against the spread); LDS reduces the 32 pixel groups; the block's
//                (count, mean, sum of squared deviations) per channel goes to the workspace.
//   bn_combine   one workgroup per channel merges the blocks' triples with the pairwise update of Chan, Golub and
//                LeVeque (mean += delta * n_b / n; M2 += M2_b + delta^2 * n_a * n_b / n): every thread a strided
//                subset in list order, then a fixed tree over the threads.
#include "bn_common.h"

namespace sbnet {

// workspace layout: float part[cap][C][2] (mean, M2), then float cnt[cap]
template <int DT>
__global__ __launch_bounds__(kBnThreads) void bn_partial(const uint4 *__restrict__ x, const int32_t *__restrict__ indices,
                                                         const int32_t *__restrict__ count, float *__restrict__ part,
                                                         float *__restrict__ cnt, BnParams p) {
    constexpr int EPV = BnElem<DT>::EPV;
    __shared__ float red[2][32][8 * EPV + 1];
    __shared__ float ref_s[8 * EPV];
    const int nact = min(*count, p.cap);
    const uint32_t items = (uint32_t)nact * (uint32_t)p.slabs;
    const int pg = threadIdx.x >> 3, k = threadIdx.x & 7;         // pixel group, vector of the slab
    for (uint32_t item = blockIdx.x; item < items; item += gridDim.x) {
        const uint32_t b = fdiv(item, p.div_slabs);
        const int slab = (int)(item - b * p.slabs);
        const int n = indices[3 * b], by = indices[3 * b + 1], bx = indices[3 * b + 2];
        const int y0 = p.g.boffset_h + by * p.g.bstride_h, x0 = p.g.boffset_w + bx * p.g.bstride_w;
        // the part of the block inside the image
        const int ylo = max(y0, 0), yhi = min(y0 + p.g.bsize_h, p.H), xlo = max(x0, 0), xhi = min(x0 + p.g.bsize_w, p.W);
        const int npx = max(yhi - ylo, 0) * max(xhi - xlo, 0);
        const int c0 = slab * p.cs + k * EPV;                     // this thread's first channel
        const bool chan_ok = c0 < p.C;
        const long long base = (long long)n * p.H * p.W * p.pix_vecs + (long long)(slab * (p.cs / EPV) + k);
        // reference value per channel: the block's first inside pixel
        if (threadIdx.x < 8) {
            float f[EPV];
#pragma unroll
            for (int e = 0; e < EPV; ++e) f[e] = 0.f;
            if (npx > 0 && chan_ok) BnElem<DT>::unpack(x[base + ((long long)ylo * p.W + xlo) * p.pix_vecs], f);
#pragma unroll
            for (int e = 0; e < EPV; ++e) ref_s[k * EPV + e] = f[e];
        }
        __syncthreads();
        float ref[EPV], s1[EPV], s2[EPV];
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            ref[e] = ref_s[k * EPV + e];
            s1[e] = s2[e] = 0.f;
        }
        for (int q0 = pg; q0 < p.hw; q0 += 32 * 4) {              // four independent loads in flight
            uint4 v[4];
            bool in[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int q = q0 + 32 * u;
                const int i = (int)fdiv((uint32_t)q, p.div_w), j = q - i * p.g.bsize_w;
                const int yy = y0 + i, xx = x0 + j;
                in[u] = chan_ok && q < p.hw && yy >= 0 && yy < p.H && xx >= 0 && xx < p.W;
                v[u] = make_uint4(0, 0, 0, 0);
                if (in[u]) v[u] = x[base + ((long long)yy * p.W + xx) * p.pix_vecs];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (in[u]) {
                    float f[EPV];
                    BnElem<DT>::unpack(v[u], f);
#pragma unroll
                    for (int e = 0; e < EPV; ++e) {
                        const float d = f[e] - ref[e];
                        s1[e] += d;
                        s2[e] = fmaf(d, d, s2[e]);
                    }
                }
        }
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            red[0][pg][k * EPV + e] = s1[e];
            red[1][pg][k * EPV + e] = s2[e];
        }
        __syncthreads();
        if (threadIdx.x < 8 * EPV) {                              // one thread per channel of the slab
            const int c = slab * p.cs + threadIdx.x;
            float a = 0.f, q2 = 0.f;
            for (int gq = 0; gq < 32; ++gq) {
                a += red[0][gq][threadIdx.x];
                q2 += red[1][gq][threadIdx.x];
            }
            if (c < p.C) {
                const float nf = (float)npx;
                const float md = npx > 0 ? a / nf : 0.f;          // mean of the deviations
                part[((size_t)b * p.C + c) * 2] = ref_s[threadIdx.x] + md;
                part[((size_t)b * p.C + c) * 2 + 1] = npx > 0 ? fmaxf(q2 - a * md, 0.f) : 0.f;
            }
            if (slab == 0 && threadIdx.x == 0) cnt[b] = (float)npx;
        }
        __syncthreads();                                          // LDS free for the next item
    }
}

// merge of two (count, mean, M2) triples; an empty side leaves the other unchanged
__device__ __forceinline__ void bn_merge(float &n, float &m, float &m2, float nb, float mb, float m2b) {
    if (nb <= 0.f) return;
    const float tot = n + nb, delta = mb - m;
    m += delta * (nb / tot);
    m2 += m2b + delta * delta * (n * nb / tot);
    n = tot;
}

// one workgroup per channel: thread t merges blocks t, t + 256, ... in that order, then the 256 partial triples are
// merged pairwise in a fixed tree
__global__ __launch_bounds__(kBnThreads) void bn_combine(const float *__restrict__ part, const float *__restrict__ cnt,
                                                         const int32_t *__restrict__ count, int cap, int C,
                                                         float *__restrict__ mean, float *__restrict__ var) {
    __shared__ float sn[kBnThreads], sm[kBnThreads], sq[kBnThreads];
    const int c = blockIdx.x;
    const int nact = min(*count, cap);
    float n = 0.f, m = 0.f, m2 = 0.f;
    for (int b = threadIdx.x; b < nact; b += kBnThreads)
        bn_merge(n, m, m2, cnt[b], part[((size_t)b * C + c) * 2], part[((size_t)b * C + c) * 2 + 1]);
    sn[threadIdx.x] = n; sm[threadIdx.x] = m; sq[threadIdx.x] = m2;
    __syncthreads();
    for (int half = kBnThreads / 2; half > 0; half >>= 1) {
        if ((int)threadIdx.x < half) {
            bn_merge(n, m, m2, sn[threadIdx.x + half], sm[threadIdx.x + half], sq[threadIdx.x + half]);
            sn[threadIdx.x] = n; sm[threadIdx.x] = m; sq[threadIdx.x] = m2;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        mean[c] = m;
        var[c] = n > 0.f ? m2 / n : 0.f;
    }
}

}  // namespace sbnet

using namespace sbnet;

extern "C" size_t sbnet_bn_stats_workspace_bytes(int cap, int C) {
    if (cap <= 0 || C <= 0) return 0;
    return ((size_t)cap * C * 2 + (size_t)cap) * sizeof(float);
}

extern "C" sbnet_status sbnet_sparse_bn_stats(const void *x, sbnet_dtype dtype, int N, int H, int W, int C,
                                              const int32_t *indices, const int32_t *count, int cap,
                                              const sbnet_geom *g, float *mean, float *var, void *workspace,
                                              size_t workspace_bytes, void *stream) {
    const char *who = "sbnet_sparse_bn_stats";
    if (!x || !indices || !count || !mean || !var) return fail(SBNET_EINVAL, "%s: null pointer", who);
    BnParams p;
    sbnet_status st = bn_fill_params(who, dtype, N, H, W, C, cap, g, &p);
    if (st != SBNET_OK) return st;
    if ((uintptr_t)x & 15) return fail(SBNET_EINVAL, "%s: x must be 16-byte aligned", who);
    if (cap > 0 && (!workspace || ((uintptr_t)workspace & 3) || workspace_bytes < sbnet_bn_stats_workspace_bytes(cap, C)))
        return fail(SBNET_EINVAL, "%s: workspace missing, misaligned or too small", who);
    hipStream_t s = (hipStream_t)stream;
    float *part = (float *)workspace;
    float *cnt = part ? part + (size_t)cap * C * 2 : nullptr;
    if (cap > 0) {
        const long long items = (long long)cap * p.slabs;
        const int grid = (int)(items < 8192 ? items : 8192);
        if (dtype == SBNET_F32)
            hipLaunchKernelGGL(bn_partial<SBNET_F32>, dim3(grid), dim3(kBnThreads), 0, s, (const uint4 *)x, indices, count, part, cnt, p);
        else if (dtype == SBNET_BF16)
            hipLaunchKernelGGL(bn_partial<SBNET_BF16>, dim3(grid), dim3(kBnThreads), 0, s, (const uint4 *)x, indices, count, part, cnt, p);
        else
            hipLaunchKernelGGL(bn_partial<SBNET_F16>, dim3(grid), dim3(kBnThreads), 0, s, (const uint4 *)x, indices, count, part, cnt, p);
    }
    hipLaunchKernelGGL(bn_combine, dim3(C), dim3(kBnThreads), 0, s, part, cnt, count, cap, C, mean, var);
    return launch_status(who);
}
