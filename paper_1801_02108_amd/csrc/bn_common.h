// Shared by the batch-norm kernels over active blocks (bn_stats.hip, bn_apply.hip): the work decomposition
// (one item = an active block x a slab of 128 bytes of channels per pixel; 8 lanes per pixel strip, 32 pixel groups
// per workgroup) and the element packing of the three storage types.
#pragma once
#include "common.h"

namespace sbnet {

constexpr int kBnThreads = 256;

struct BnParams {
    sbnet_geom g;
    int H, W, C, cap;
    int slabs, cs;               // slabs per pixel, channels per full slab (128 bytes)
    uint32_t pix_vecs;           // 16-byte vectors per pixel
    int hw;                      // pixels per block
    FastDiv div_slabs, div_w;
};

template <int DT> struct BnElem;
template <> struct BnElem<SBNET_F32> {
    static constexpr int EPV = 4;
    static __device__ __forceinline__ void unpack(const uint4 &v, float *f) {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    }
};
template <> struct BnElem<SBNET_BF16> {
    static constexpr int EPV = 8;
    static __device__ __forceinline__ void unpack(const uint4 &v, float *f) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = bf16_bits_to_float(w[i] & 0xffffu);
            f[2 * i + 1] = bf16_bits_to_float(w[i] >> 16);
        }
    }
};
template <> struct BnElem<SBNET_F16> {
    static constexpr int EPV = 8;
    static __device__ __forceinline__ void unpack(const uint4 &v, float *f) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            union { _Float16 h[2]; uint32_t u; } x;
            x.u = w[i];
            f[2 * i] = (float)x.h[0];
            f[2 * i + 1] = (float)x.h[1];
        }
    }
};

// fp32 -> storage type, round to nearest even
template <int DT>
__device__ __forceinline__ uint4 bn_pack(const float *f) {
    if (DT == SBNET_F32) return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (DT == SBNET_BF16) {
            w[i] = float_to_bf16_bits(f[2 * i]) | (float_to_bf16_bits(f[2 * i + 1]) << 16);
        } else {
            union { _Float16 h[2]; uint32_t u; } x;
            x.h[0] = (_Float16)f[2 * i];
            x.h[1] = (_Float16)f[2 * i + 1];
            w[i] = x.u;
        }
    }
    return make_uint4(w[0], w[1], w[2], w[3]);
}

inline sbnet_status bn_fill_params(const char *who, sbnet_dtype dtype, int N, int H, int W, int C, int cap,
                                   const sbnet_geom *g, BnParams *p) {
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || cap < 0) return fail(SBNET_EINVAL, "%s: bad sizes", who);
    if (!geom_ok(g)) return fail(SBNET_EINVAL, "%s: bad geometry", who);
    if (!is_float_dtype(dtype)) return fail(SBNET_EUNSUPPORTED, "%s: dtype must be f32, bf16 or f16", who);
    if (g->bstride_h < g->bsize_h || g->bstride_w < g->bsize_w)
        return fail(SBNET_EINVAL, "%s: blocks must not overlap (every pixel counts once)", who);
    const int es = elem_bytes(dtype);
    if ((long long)C * es % 16) return fail(SBNET_EUNSUPPORTED, "%s: a pixel's channels must fill 16-byte vectors", who);
    if ((long long)g->bsize_h * g->bsize_w >= (1LL << 24))
        return fail(SBNET_EUNSUPPORTED, "%s: block too large (pixel counts are kept in fp32)", who);
    p->g = *g;
    p->H = H; p->W = W; p->C = C; p->cap = cap;
    p->cs = 128 / es;
    p->slabs = (C + p->cs - 1) / p->cs;
    p->pix_vecs = (uint32_t)(C * es / 16);
    p->hw = g->bsize_h * g->bsize_w;
    if ((long long)cap * p->slabs >= (1LL << 31)) return fail(SBNET_EUNSUPPORTED, "%s: too many work items", who);
    p->div_slabs = make_fastdiv((uint32_t)p->slabs);
    p->div_w = make_fastdiv((uint32_t)g->bsize_w);
    return SBNET_OK;
}

}  // namespace sbnet
