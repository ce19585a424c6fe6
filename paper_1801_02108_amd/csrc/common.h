// Shared host-side plumbing of the gfx950 tiled sparse convolution library: error
// reporting, argument checks, element-type helpers.  No arithmetic of the method lives here.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>

#include "../../include/sbnet.h"

namespace sbnet {

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

// bf16 <-> fp32 on the device (round to nearest even; NaN kept quiet)
__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

}  // namespace sbnet
