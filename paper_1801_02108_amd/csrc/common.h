// Shared host-side plumbing of the gfx950 tiled sparse convolution library: error
// reporting, argument checks, element-type helpers.  No arithmetic of the method lives here.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>

#include "../../include/sbnet.h"

namespace sbnet {

// the compute-tile choices in force (sbnet_set_tuning), read when a call is enqueued
sbnet_tuning tuning();

// thread-local text behind sbnet_last_error()
char *error_buffer();
sbnet_status fail(sbnet_status code, const char *fmt, ...);

inline int elem_bytes(sbnet_dtype dt) {
    switch (dt) {
        case SBNET_F32: return 4;
        case SBNET_BF16: return 2;
        case SBNET_F16: return 2;
        case SBNET_U8: return 1;
    }
    return 0;
}

inline bool is_float_dtype(sbnet_dtype dt) { return dt == SBNET_F32 || dt == SBNET_BF16 || dt == SBNET_F16; }

inline bool geom_ok(const sbnet_geom *g) {
    return g && g->bsize_h > 0 && g->bsize_w > 0 && g->bstride_h > 0 && g->bstride_w > 0 &&
           g->bcount_h > 0 && g->bcount_w > 0;
}

// reduce_mask.hip, pass 1 of the small-grid path, also used by the fused consumers: one flag byte per block in
// lexicographic (n, by, bx) order.  `flags` must hold N * bcount_h * bcount_w bytes rounded up to 16.
bool mask_flag_path(int N, const sbnet_geom *g);
sbnet_status mask_to_flags(const char *who, const void *mask, sbnet_dtype mdt, int N, int H, int W, const sbnet_geom *g,
                           sbnet_pool pool, float threshold, uint8_t *flags, hipStream_t s);

// pass 2 of the same path: flags -> index list and count
sbnet_status flags_to_indices(const char *who, const uint8_t *flags, int N, const sbnet_geom *g, int32_t *indices,
                              int32_t *count, int cap, hipStream_t s);

// bottleneck.hip: the downsampling residual unit (stride 2, projected shortcut) in one launch, for the shapes it
// serves; SBNET_EUNSUPPORTED otherwise.  Arguments as sbnet_sparse_unit, already validated by it.
sbnet_status unit_down_try(const char *who, const void *x, sbnet_dtype dt, int N, int H, int W, int C, int Cm, int CO,
                           const int32_t *indices, const int32_t *count, int cap, const sbnet_geom *g_in,
                           const sbnet_geom *g_out, const void *w1, const float *b1, const void *w2, const float *b2,
                           const void *w3, const float *b3, const void *ws, const float *bs, void *y, int Ho, int Wo,
                           void *stream);

// do the byte ranges [a, a + a_bytes) and [b, b + b_bytes) share a byte?
inline bool ranges_overlap(const void *a, size_t a_bytes, const void *b, size_t b_bytes) {
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + b_bytes && b0 < a0 + a_bytes;
}

inline sbnet_status launch_status(const char *what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(SBNET_EHIP, "%s: %s", what, hipGetErrorString(e));
    return SBNET_OK;
}

// Exact unsigned division by a runtime constant d (1 <= d < 2^31) for numerators below 2^31:
// q = (n * m) >> 32 >> s with m = ceil(2^(32+s) / d), s = ceil(log2 d).
struct FastDiv {
    uint32_t m, s, d;
};
inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f;
    f.d = d;
    uint32_t s = 0;
    while ((1u << s) < d) ++s;
    f.s = s;
    f.m = (uint32_t)(((((uint64_t)1 << s) - d) << 32) / d + 1);
    return f;
}
__device__ __forceinline__ uint32_t fdiv(uint32_t n, const FastDiv f) {
    // round-up method: q = (t + ((n - t) >> 1)) >> (s - 1), t = mulhi(n, m); valid for all n < 2^32
    uint32_t t = __umulhi(n, f.m);
    return f.s == 0 ? n : (t + ((n - t) >> 1)) >> (f.s - 1);
}

// Inclusive prefix sum of a non-negative int over the 64 lanes (lane 63: the total): four shifts inside the
// rows of 16 lanes, then the row totals are passed on to the next row and to the upper half.  Cross-lane
// moves in the VALU's data path, no LDS round trips; lanes without a source read 0.
__device__ __forceinline__ int wave_inclusive_sum(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
    return v;
}

// 16-bit mask of the non-zero bytes among the first `valid` (0..16) bytes of q (bit i = byte i)
__device__ __forceinline__ uint32_t nonzero_bytes16(uint4 q, int valid) {
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
    uint32_t bits = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        uint32_t t = w[k];
        t |= t >> 4; t |= t >> 2; t |= t >> 1;
        t &= 0x01010101u;                                        // bit 0 of every byte: byte != 0
        t = (t | (t >> 7) | (t >> 14) | (t >> 21)) & 0xfu;       // gathered into four neighbouring bits
        bits |= t << (4 * k);
    }
    return valid >= 16 ? bits : (valid <= 0 ? 0u : bits & ((1u << valid) - 1u));
}

// bf16 <-> fp32 on the device (round to nearest even; NaN kept quiet)
__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

}  // namespace sbnet
