// 8-bit floating-point variant of the tile convolution (Sec. 3.2 of arXiv 1801.02108 computes the convolution between
// gather and scatter in whatever precision the dense engine offers; the paper names none).  Tiles and weights are
// stored as FP8 E4M3 (the OCP "e4m3fn" encoding: 4 exponent bits with bias 7, 3 mantissa bits, no infinities, largest
// finite value 448), products are exact and summed in fp32 on the matrix cores, and the result
//   out = act(out_scale * sum + bias)
// leaves as BF16 (out_scale undoes the scales the caller quantised inputs and weights with).
//
//   f8_quantize     out = e4m3(clamp(x * scale, -448, 448)), round to nearest even, for any F32 / BF16 / F16 buffer
//                   (a gathered tile stack, a weight array).
//   f8_pack_weights [kh][kw][Cin][Cout] bytes -> MFMA operand order (below).
//   conv_f8_mfma    implicit GEMM as conv_mfma does it for 16-bit types: a workgroup computes 256 (or 64) output
//                   pixels x 64 output channels, input rows staged in LDS in channel chunks, weight fragments from L2
//                   through a ring a few k-steps ahead, 16x16x32 FP8 MFMA (8 bytes per lane and operand).
//
// Packed weights: byte (((ng*KS + ks)*4 + nb)*64 + lane)*8 + e holds w[tap][c][o] with ks = tap*(CinP/32) + c/32,
// c = (ks % (CinP/32))*32 + (lane/16)*8 + e and o = ng*64 + (nb/2)*32 + ((lane%16)/4)*8 + (nb%2)*4 + (lane%16)%4 (zero
// where c >= Cin or o >= Cout): with this permutation of o the accumulator fragments nb = 2h, 2h+1 of a lane hold 8
// consecutive channels, one 16-byte BF16 store.
#include <hip/hip_runtime.h>

#include "conv_common.h"

namespace sbnet {
namespace {

constexpr int kNB8 = 4;      // 16-channel blocks per wave (64 output channels per workgroup)
constexpr int kWD8 = 4;      // k-steps of weight fragments in flight
constexpr int kStage8 = 8;   // input vectors in flight per thread while a chunk is staged

struct F8Params {
    const uint8_t *in;       // [cap][th][tw][Cin]
    void *out;               // [cap][oh][ow][Cout] bf16
    const uint8_t *w;        // packed
    const float *bias;
    const int32_t *count;
    float out_scale;
    int cap, th, tw, oh, ow, Cin, Cout, kh, kw, sh, sw, relu;
    int CinP, CC, nchunks, mpasses, ngroups;
    FastDiv div_ow, div_tw, div_cv, div_cv_last, div_pn, div_ng;
};

// fp32 -> e4m3fn bits, round to nearest even, saturating; NaN -> 0x7f
__device__ __forceinline__ uint32_t f32_to_e4m3(float x) {
    if (x != x) return 0x7fu;
    const uint32_t sign = (__float_as_uint(x) >> 24) & 0x80u;
    float a = fminf(fabsf(x), 448.f);
    // below 2^-6 the format is subnormal with a fixed step of 2^-9: round the value in units of that step
    if (a < 0.015625f) {                                         // 2^-6
        const float q = rintf(a * 512.f);                        // multiples of 2^-9, ties to even
        return sign | (uint32_t)q;                               // q = 8 is the smallest normal (0x08)
    }
    uint32_t u = __float_as_uint(a);
    u += 0x7ffffu + ((u >> 20) & 1u);                            // round the 23-bit mantissa to 3 bits, ties to even
    const uint32_t e = (u >> 23) - 127u + 7u, m = (u >> 20) & 7u;
    return sign | (e << 3) | m;                                  // a <= 448 keeps e <= 15 and excludes 0x7f
}

template <int DT>
__device__ __forceinline__ float f8_source(const void *x, size_t i) {
    if (DT == SBNET_F32) return ((const float *)x)[i];
    if (DT == SBNET_BF16) return bf16_bits_to_float(((const uint16_t *)x)[i]);
    return unpack_lo<SBNET_F16>(((const uint16_t *)x)[i]);
}

// eight elements per thread and step (16 or 32 bytes in, 8 bytes out) where the buffers allow it, single elements
// for the tail
template <int DT>
__global__ __launch_bounds__(256) void f8_quantize(const void *__restrict__ x, uint8_t *__restrict__ out, size_t elems, float scale,
                                                   int vector_ok) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const size_t groups = vector_ok ? elems / 8 : 0;
    for (size_t gi = (size_t)blockIdx.x * blockDim.x + threadIdx.x; gi < groups; gi += stride) {
        float v[8];
        if (DT == SBNET_F32) {
            const float4 a = ((const float4 *)x)[2 * gi], b = ((const float4 *)x)[2 * gi + 1];
            v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
        } else {
            const uint4 a = ((const uint4 *)x)[gi];
            const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                v[2 * k] = unpack_lo<DT>(w[k]);
                v[2 * k + 1] = unpack_hi<DT>(w[k]);
            }
        }
        uint32_t lo = 0, hi = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            lo |= f32_to_e4m3(v[k] * scale) << (8 * k);
            hi |= f32_to_e4m3(v[4 + k] * scale) << (8 * k);
        }
        ((uint2 *)out)[gi] = make_uint2(lo, hi);
    }
    for (size_t i = groups * 8 + (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < elems; i += stride)
        out[i] = (uint8_t)f32_to_e4m3(f8_source<DT>(x, i) * scale);
}

__global__ void f8_pack_weights(const uint8_t *__restrict__ w, uint8_t *__restrict__ packed, int taps, int Cin, int Cout, int CinP,
                                int ngroups) {
    const int KS = taps * (CinP / 32);
    const size_t total = (size_t)ngroups * KS * kNB8 * 64 * 8;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
        const int e = (int)(idx & 7);
        const int lane = (int)((idx >> 3) & 63);
        const int nb = (int)((idx >> 9) & 3);
        const size_t rest = idx >> 11;
        const int ks = (int)(rest % KS), ng = (int)(rest / KS);
        const int tap = ks / (CinP / 32);
        const int c = (ks % (CinP / 32)) * 32 + (lane >> 4) * 8 + e;
        const int rho = lane & 15;
        const int o = ng * 64 + (nb >> 1) * 32 + (rho >> 2) * 8 + (nb & 1) * 4 + (rho & 3);
        packed[idx] = (c < Cin && o < Cout) ? w[((size_t)tap * Cin + c) * Cout + o] : (uint8_t)0;
    }
}

__device__ __forceinline__ f32x4 mfma16x16x32_f8(uint2 a, uint2 b, f32x4 c) {
    const long la = (long)(((unsigned long long)a.y << 32) | a.x), lb = (long)(((unsigned long long)b.y << 32) | b.x);
    return __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(la, lb, c, 0, 0, 0);
}

template <int kMB>
__global__ __launch_bounds__(256) void conv_f8_mfma(F8Params p) {
    constexpr int PP = 64 * kMB;                // output pixels per pass
    extern __shared__ __align__(16) unsigned char lds[];
    uint16_t *out = (uint16_t *)p.out;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = lane >> 4, l16 = lane & 15;
    const int nact = min(*p.count, p.cap);
    const int M = p.oh * p.ow;
    const int pix_stride = p.CC + 8;            // bytes between pixels in LDS: 8-byte reads of 16 pixels hit 32 banks
    const int c32_total = p.CinP / 32;
    const int KS = p.kh * p.kw * c32_total;
    const uint32_t per_tile = (uint32_t)p.mpasses * p.ngroups;
    const uint32_t items = (uint32_t)nact * per_tile;

    for (uint32_t item = blockIdx.x; item < items; item += gridDim.x) {
        const uint32_t b = fdiv(item, p.div_pn);
        const uint32_t rest = item - b * per_tile;
        const int pass = (int)fdiv(rest, p.div_ng);
        const int ng = (int)rest - pass * p.ngroups;

        // output pixels of this pass and the input rows they need
        const int p_lo = pass * PP, p_hi = min(p_lo + PP, M);
        const int i_lo = (int)fdiv(p_lo, p.div_ow), i_hi = (int)fdiv(p_hi - 1, p.div_ow);
        const int r_lo = i_lo * p.sh;
        const int nrows = (i_hi - i_lo) * p.sh + p.kh;

        int xbase[kMB], pixel[kMB];
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb) {
            int px = p_lo + (wave * kMB + mb) * 16 + l16;
            pixel[mb] = px;
            px = min(px, M - 1);
            const int i = (int)fdiv(px, p.div_ow), j = px - i * p.ow;
            xbase[mb] = ((i * p.sh - r_lo) * p.tw + j * p.sw) * pix_stride + q * 8;
        }

        f32x4 acc[kMB][kNB8];
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
            for (int nb = 0; nb < kNB8; ++nb) acc[mb][nb] = (f32x4){0.f, 0.f, 0.f, 0.f};

        for (int chunk = 0; chunk < p.nchunks; ++chunk) {
            const int c0 = chunk * p.CC;
            const int cc = min(p.CC, p.CinP - c0);      // channels in this chunk (multiple of 32)
            const int cv = cc >> 4;                     // 16-byte vectors (16 channels) per pixel
            const FastDiv dcv = (chunk == p.nchunks - 1) ? p.div_cv_last : p.div_cv;
            __syncthreads();                            // previous chunk / item fully consumed
            const uint32_t nvec = (uint32_t)nrows * p.tw * cv;
            for (uint32_t v0 = threadIdx.x; v0 < nvec; v0 += 256 * kStage8) {
                uint4 val[kStage8];
                uint32_t dst[kStage8];
#pragma unroll
                for (int u = 0; u < kStage8; ++u) {
                    const uint32_t v = v0 + u * 256;
                    const uint32_t px = fdiv(v, dcv);
                    const int c16 = (int)(v - px * cv);
                    const int row = (int)fdiv(px, p.div_tw), col = (int)px - row * p.tw;
                    const int c = c0 + c16 * 16;
                    val[u] = make_uint4(0, 0, 0, 0);
                    dst[u] = px * pix_stride + c16 * 16;
                    if (v < nvec && c < p.Cin)          // Cin % 16 == 0: a vector is all in or all out
                        val[u] = *(const uint4 *)(p.in + (((size_t)b * p.th + r_lo + row) * p.tw + col) * p.Cin + c);
                }
#pragma unroll
                for (int u = 0; u < kStage8; ++u)
                    if (v0 + u * 256 < nvec) {          // the pixel stride is a multiple of 8 bytes, not of 16
                        *(uint2 *)(lds + dst[u]) = make_uint2(val[u].x, val[u].y);
                        *(uint2 *)(lds + dst[u] + 8) = make_uint2(val[u].z, val[u].w);
                    }
            }
            __syncthreads();

            // k loop over (tap row, tap column, 32-channel step); weight fragments through a ring of kWD8 steps
            const int steps = cc >> 5;
            const int nit = p.kh * p.kw * steps;
            const uint2 *wbase = (const uint2 *)p.w + ((size_t)ng * KS + (c0 >> 5)) * kNB8 * 64 + lane;
            int lt = 0, lst = 0;                       // request cursor: tap, channel step
            uint2 ring[kWD8][kNB8];
            auto request = [&](int slot) __attribute__((always_inline)) {
                const uint2 *wp = wbase + ((size_t)(lt * c32_total + lst) * kNB8) * 64;
#pragma unroll
                for (int nb = 0; nb < kNB8; ++nb) ring[slot][nb] = wp[(size_t)nb * 64];
                const bool last = (lt == p.kh * p.kw - 1) && (lst == steps - 1);   // never past the last step
                if (!last) {
                    if (++lst == steps) { lst = 0; ++lt; }
                }
            };
            int r = 0, t = 0, st = 0;                  // use cursor: tap row, tap column, channel step
            auto one_step = [&](int slot) __attribute__((always_inline)) {
                const int off = (r * p.tw + t) * pix_stride + st * 32;
                uint2 xf[kMB];
#pragma unroll
                for (int mb = 0; mb < kMB; ++mb) xf[mb] = *(const uint2 *)(lds + xbase[mb] + off);
#pragma unroll
                for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
                    for (int nb = 0; nb < kNB8; ++nb) acc[mb][nb] = mfma16x16x32_f8(ring[slot][nb], xf[mb], acc[mb][nb]);
                if (++st == steps) { st = 0; if (++t == p.kw) { t = 0; ++r; } }
            };
#pragma unroll
            for (int u = 0; u < kWD8; ++u) request(u);
            int it = 0;
            for (; it + kWD8 <= nit; it += kWD8) {
#pragma unroll
                for (int u = 0; u < kWD8; ++u) {
                    one_step(u);
                    request(u);
                }
            }
#pragma unroll
            for (int u = 0; u < kWD8 - 1; ++u)
                if (it + u < nit) one_step(u);
        }

        // epilogue: lane holds channels ng*64 + h*32 + q*8 + [0,8), h = 0,1, of pixel (mb, l16)
        float bias[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const int o = ng * 64 + (k >> 3) * 32 + q * 8 + (k & 7);
            bias[k] = (p.bias && o < p.Cout) ? p.bias[o] : 0.f;
        }
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb) {
            const int px = pixel[mb];
            if (px >= p_hi) continue;
            uint16_t *dst = out + ((size_t)b * M + px) * p.Cout;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int o0 = ng * 64 + half * 32 + q * 8;
                if (o0 >= p.Cout) continue;   // Cout % 8 == 0: a vector is all in or all out
                float v[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const float a = fmaf(acc[mb][half * 2 + (k >> 2)][k & 3], p.out_scale, bias[half * 8 + k]);
                    v[k] = p.relu ? fmaxf(a, 0.f) : a;
                }
                *(uint4 *)(dst + o0) = make_uint4(pack2<SBNET_BF16>(v[0], v[1]), pack2<SBNET_BF16>(v[2], v[3]),
                                                  pack2<SBNET_BF16>(v[4], v[5]), pack2<SBNET_BF16>(v[6], v[7]));
            }
        }
    }
}

size_t f8_packed_bytes(int kh, int kw, int Cin, int Cout) {
    const size_t CinP = (size_t)(Cin + 31) / 32 * 32, CoutP = (size_t)(Cout + 63) / 64 * 64;
    return (size_t)kh * kw * CinP * CoutP;
}

}  // namespace
}  // namespace sbnet

using namespace sbnet;

extern "C" sbnet_status sbnet_quantize_f8(const void *x, sbnet_dtype dtype, size_t elems, float scale, void *out, void *stream) {
    const char *who = "sbnet_quantize_f8";
    if (!x || !out) return fail(SBNET_EINVAL, "%s: null pointer", who);
    if (!is_float_dtype(dtype)) return fail(SBNET_EUNSUPPORTED, "%s: dtype must be f32, bf16 or f16", who);
    if (!(scale > 0.f) || scale * 0.f != 0.f) return fail(SBNET_EINVAL, "%s: scale must be positive and finite", who);
    if (elems == 0) return SBNET_OK;
    const int vector_ok = (((uintptr_t)x & 15) == 0 && ((uintptr_t)out & 7) == 0) ? 1 : 0;
    const size_t want = (elems / 8 + 255) / 256 + 1;
    const int grid = (int)(want > 4096 ? 4096 : want);
    hipStream_t s = (hipStream_t)stream;
    if (dtype == SBNET_F32) hipLaunchKernelGGL(f8_quantize<SBNET_F32>, dim3(grid), dim3(256), 0, s, x, (uint8_t *)out, elems, scale, vector_ok);
    else if (dtype == SBNET_BF16) hipLaunchKernelGGL(f8_quantize<SBNET_BF16>, dim3(grid), dim3(256), 0, s, x, (uint8_t *)out, elems, scale, vector_ok);
    else hipLaunchKernelGGL(f8_quantize<SBNET_F16>, dim3(grid), dim3(256), 0, s, x, (uint8_t *)out, elems, scale, vector_ok);
    return launch_status(who);
}

extern "C" sbnet_status sbnet_pack_weights_f8(const void *w_hwio_f8, int kh, int kw, int Cin, int Cout, void *w_packed,
                                              size_t *bytes, void *stream) {
    const char *who = "sbnet_pack_weights_f8";
    if (kh <= 0 || kw <= 0 || Cin <= 0 || Cout <= 0) return fail(SBNET_EINVAL, "%s: bad sizes", who);
    const size_t total = f8_packed_bytes(kh, kw, Cin, Cout);
    if (bytes) *bytes = total;
    if (!w_packed) {
        if (!bytes) return fail(SBNET_EINVAL, "%s: nothing to do", who);
        return SBNET_OK;
    }
    if (!w_hwio_f8) return fail(SBNET_EINVAL, "%s: null weights", who);
    const int grid = (int)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    hipLaunchKernelGGL(f8_pack_weights, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const uint8_t *)w_hwio_f8,
                       (uint8_t *)w_packed, kh * kw, Cin, Cout, (Cin + 31) / 32 * 32, (Cout + 63) / 64);
    return launch_status(who);
}

extern "C" sbnet_status sbnet_conv_on_tiles_f8(const void *tiles_in_f8, const int32_t *count, int cap, int th, int tw, int Cin,
                                               const void *w_packed_f8, const float *bias, int kh, int kw, int sh, int sw,
                                               int Cout, int relu, float out_scale, void *tiles_out_bf16, void *stream) {
    const char *who = "sbnet_conv_on_tiles_f8";
    if (!tiles_in_f8 || !count || !w_packed_f8 || !tiles_out_bf16) return fail(SBNET_EINVAL, "%s: null pointer", who);
    if (cap < 0 || th <= 0 || tw <= 0 || Cin <= 0 || Cout <= 0 || kh <= 0 || kw <= 0 || sh <= 0 || sw <= 0 || th < kh || tw < kw)
        return fail(SBNET_EINVAL, "%s: bad sizes", who);
    if (Cin % 16 || Cout % 8) return fail(SBNET_EUNSUPPORTED, "%s: Cin must be a multiple of 16 and Cout of 8", who);
    if (((uintptr_t)tiles_in_f8 | (uintptr_t)tiles_out_bf16 | (uintptr_t)w_packed_f8) & 15)
        return fail(SBNET_EINVAL, "%s: pointers must be 16-byte aligned", who);
    if (!(out_scale == out_scale) || out_scale * 0.f != 0.f) return fail(SBNET_EINVAL, "%s: out_scale must be finite", who);
    if (cap == 0) return SBNET_OK;
    F8Params p = {};
    p.in = (const uint8_t *)tiles_in_f8; p.out = tiles_out_bf16; p.w = (const uint8_t *)w_packed_f8; p.bias = bias;
    p.count = count; p.out_scale = out_scale; p.cap = cap;
    p.th = th; p.tw = tw; p.Cin = Cin; p.Cout = Cout; p.kh = kh; p.kw = kw; p.sh = sh; p.sw = sw; p.relu = relu ? 1 : 0;
    p.oh = (th - kh) / sh + 1;
    p.ow = (tw - kw) / sw + 1;
    const long long M = (long long)p.oh * p.ow;
    if (M * Cout >= (1LL << 31) || (long long)th * tw * Cin >= (1LL << 31)) return fail(SBNET_EUNSUPPORTED, "%s: tile too large", who);
    p.div_ow = make_fastdiv(p.ow);
    p.div_tw = make_fastdiv(p.tw);
    p.CinP = (Cin + 31) / 32 * 32;
    p.ngroups = (Cout + 63) / 64;
    // 64-pixel passes when even the caller's bound on the active tiles leaves half the CUs without a 256-pixel item
    const int PP = ((long long)cap * ((M + 255) / 256) * p.ngroups < 128) ? 64 : 256;
    p.mpasses = (int)((M + PP - 1) / PP);
    int out_rows = (PP + p.ow - 1) / p.ow + ((PP % p.ow) ? 1 : 0);
    if (out_rows > p.oh) out_rows = p.oh;
    int lds_rows = (out_rows - 1) * sh + kh;
    if (lds_rows > th) lds_rows = th;
    const long long px = (long long)lds_rows * tw;
    int CC = p.CinP;
    while (CC > 32 && px * (CC + 8) > 64 * 1024) CC -= 32;
    const long long lds_bytes = px * (CC + 8);
    if (lds_bytes > 160 * 1024) return fail(SBNET_EUNSUPPORTED, "%s: tile rows do not fit in LDS", who);
    p.CC = CC;
    p.nchunks = (p.CinP + CC - 1) / CC;
    p.div_cv = make_fastdiv(CC / 16);
    const int last_c = p.CinP - (p.nchunks - 1) * CC;
    p.div_cv_last = make_fastdiv(last_c / 16 > 0 ? last_c / 16 : 1);
    p.div_pn = make_fastdiv((uint32_t)p.mpasses * p.ngroups);
    p.div_ng = make_fastdiv(p.ngroups);
    const long long items = (long long)cap * p.mpasses * p.ngroups;
    if (items >= (1LL << 31)) return fail(SBNET_EUNSUPPORTED, "%s: too many work items", who);
    const int grid = (int)(items < 8192 ? items : 8192);
    hipStream_t s = (hipStream_t)stream;
    if (PP == 256) {
        if (lds_bytes > 48 * 1024)
            (void)hipFuncSetAttribute((const void *)conv_f8_mfma<4>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        hipLaunchKernelGGL(conv_f8_mfma<4>, dim3(grid), dim3(256), (size_t)lds_bytes, s, p);
    } else {
        if (lds_bytes > 48 * 1024)
            (void)hipFuncSetAttribute((const void *)conv_f8_mfma<1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        hipLaunchKernelGGL(conv_f8_mfma<1>, dim3(grid), dim3(256), (size_t)lds_bytes, s, p);
    }
    return launch_status(who);
}
