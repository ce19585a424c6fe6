// Convolution on gathered tiles and its fused form (Fig. 1 and Sec. 3.2 of arXiv 1801.02108):
// a regular unpadded convolution runs on every active tile; in the fused entry point the
// gather of the input tile and the scatter (or scatter-add, Sec. 3.4) of the output block
// happen inside the same kernel, so the tile stacks never reach HBM.
//
// Two kernels here, two more behind conv16_try / conv3_try (conv16.hip: 3x3 stride 1 on tiles whose sides are
// multiples of 16 with 32 or 64 input channels; conv3.hip: every other 3x3 case the matrix cores can take), which
// are asked first:
//   conv_direct  any shape, any of f32/bf16/f16: one thread per output element, fp32 FMA chain.
//                Used for f32 (there is no fp32 MFMA worth using at these sizes) and for channel
//                counts the MFMA path does not take.
//   conv_mfma    bf16/f16 with Cin % 8 == 0 and Cout % 8 == 0, kernel sizes other than 3x3 (and 3x3 tiles too
//                large for the other kernels' LDS plans): implicit GEMM on the matrix cores.
//                Per workgroup: up to 256 output pixels x 64 output channels, fp32 accumulators in
//                registers.  The input rows those pixels need are staged in LDS in channel chunks
//                (pixel stride padded by 16 B so the 16-byte operand reads of 16 neighbouring pixels
//                fall in distinct banks); the nine taps are nine uniform offsets into that one LDS
//                copy, so no im2col matrix is ever materialised (the lowering the paper argues
//                against in Sec. 2).  Weights are pre-packed into MFMA operand order and stream from
//                L2 as one coalesced 1 KB read per fragment.
//                The weights are the MFMA "A" operand (rows = output channels) and the pixels the
//                "B" operand (columns = pixels), so each lane ends up with 16 consecutive output
//                channels of one pixel and writes them as two 16-byte NHWC stores.
#include "conv_common.h"

namespace sbnet {

// ------------------------------------------------------------------------------------------
// direct kernel
// ------------------------------------------------------------------------------------------
template <int DT, bool FUSED>
__global__ __launch_bounds__(256) void conv_direct(ConvParams p) {
    typedef typename Elem<DT>::T T;
    const T *in = (const T *)p.in;
    T *out = (T *)p.out;
    const T *w = (const T *)p.w;  // HWIO
    const int nact = min(*p.count, p.cap);
    const uint32_t per_tile = (uint32_t)p.oh * p.ow * p.Cout;
    const FastDiv div_cout = p.div_cv;  // reused: divides by Cout in this kernel
    for (int b = blockIdx.y; b < nact; b += gridDim.y) {
        int n = 0, y0 = 0, x0 = 0, oy0 = 0, ox0 = 0;
        if (FUSED) {
            n = p.indices[3 * b];
            const int by = p.indices[3 * b + 1], bx = p.indices[3 * b + 2];
            y0 = p.g_in.boffset_h + by * p.g_in.bstride_h;
            x0 = p.g_in.boffset_w + bx * p.g_in.bstride_w;
            oy0 = p.g_out.boffset_h + by * p.g_out.bstride_h;
            ox0 = p.g_out.boffset_w + bx * p.g_out.bstride_w;
        }
        for (uint32_t e = blockIdx.x * 256 + threadIdx.x; e < per_tile; e += gridDim.x * 256) {
            const uint32_t pix = fdiv(e, div_cout);
            const int o = (int)(e - pix * p.Cout);
            const int i = (int)fdiv(pix, p.div_ow), j = (int)pix - i * p.ow;
            float acc = p.bias ? p.bias[o] : 0.f;
            for (int r = 0; r < p.kh; ++r)
                for (int t = 0; t < p.kw; ++t) {
                    const int yy = i * p.sh + r, xx = j * p.sw + t;
                    const T *src;
                    if (FUSED) {
                        const int gy = y0 + yy, gx = x0 + xx;
                        if (gy < 0 || gy >= p.H || gx < 0 || gx >= p.W) continue;  // zero padding
                        src = in + (((size_t)n * p.H + gy) * p.W + gx) * p.Cin;
                    } else {
                        src = in + (((size_t)b * p.th + yy) * p.tw + xx) * p.Cin;
                    }
                    const T *wp = w + ((size_t)(r * p.kw + t) * p.Cin) * p.Cout + o;
                    for (int c = 0; c < p.Cin; ++c) acc = fmaf(Elem<DT>::load(src + c), Elem<DT>::load(wp + (size_t)c * p.Cout), acc);
                }
            if (p.relu) acc = fmaxf(acc, 0.f);
            if (FUSED) {
                const int gy = oy0 + i, gx = ox0 + j;
                if (gy < 0 || gy >= p.Ho || gx < 0 || gx >= p.Wo) continue;
                T *dst = out + (((size_t)n * p.Ho + gy) * p.Wo + gx) * p.Cout + o;
                if (p.add) acc += Elem<DT>::load(dst);
                Elem<DT>::store(dst, acc);
            } else {
                Elem<DT>::store(out + ((size_t)b * p.oh * p.ow + pix) * p.Cout + o, acc);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// MFMA kernel
// ------------------------------------------------------------------------------------------
// 16-pixel blocks per wave is a template parameter of conv_mfma (MB): 4 (256 output pixels per workgroup) or, for
// problems with too few work items to occupy the device, 1 (64 pixels: four times the work items, a quarter of
// the staging and matrix work in each)
constexpr int kNB = 4;  // 16-channel blocks per wave (64 output channels per workgroup)
constexpr int kWD = 4;  // steps of weight fragments in flight ahead of the matrix work
constexpr int kStage = 12;  // input vectors in flight per thread while a chunk is staged into LDS

// Where the weight of (tap, input channel c, output channel o) of the convolution being packed for lies in the
// caller's array.  Plain: that array is this convolution's own [taps][Cin][Cout].  Transposed: the array is the
// [taps][Cout][Cin] filter bank of the forward convolution whose data gradient this convolution computes; the
// gradient correlates with the taps mirrored and the two channel roles exchanged.
__device__ __forceinline__ size_t weight_index(int tap, int c, int o, int taps, int Cin, int Cout, int transposed) {
    return transposed ? ((size_t)(taps - 1 - tap) * Cout + o) * Cin + c : ((size_t)tap * Cin + c) * Cout + o;
}

// Weight packing for conv_mfma.  Packed element (((ng*KS + ks)*4 + nb)*64 + lane)*8 + e holds
// w[tap][c][o] with ks = tap*(CinP/32) + c/32, c = (ks % (CinP/32))*32 + (lane/16)*8 + e and
// o = ng*64 + (nb/2)*32 + ((lane%16)/4)*8 + (nb%2)*4 + (lane%16)%4, zero where c >= Cin or
// o >= Cout.  With this permutation of o the accumulator fragments nb = 2h, 2h+1 of a lane hold 8
// consecutive channels (one 16-byte store), and the four lanes sharing a pixel cover 32
// consecutive channels per half h.
template <typename T>
__global__ void pack_mfma_weights(const T *__restrict__ w, T *__restrict__ packed, int taps, int Cin, int Cout,
                                  int CinP, int ngroups, int transposed) {
    const int KS = taps * (CinP / 32);
    const size_t total = (size_t)ngroups * KS * kNB * 64 * 8;
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
        T v = 0;
        if (c < Cin && o < Cout) v = w[weight_index(tap, c, o, taps, Cin, Cout, transposed)];
        packed[idx] = v;
    }
}

// Second copy of the weights in 32x32x16 operand order (used by the register-stationary 3x3
// kernel).  Packed element (((ng*KS + ks)*2 + nb)*64 + lane)*8 + e holds w[tap][c][o] with
// ks = tap*(CinP/16) + c/16, c = (ks % (CinP/16))*16 + (lane/32)*8 + e and, with rho = lane%32,
// o = ng*64 + nb*32 + ((rho/4)%2)*16 + (rho/8)*4 + rho%4: the 16 accumulator registers of a lane
// then hold 16 consecutive output channels.
template <typename T>
__global__ void pack_mfma32_weights(const T *__restrict__ w, T *__restrict__ packed, int taps, int Cin, int Cout,
                                    int CinP, int ngroups, int transposed) {
    const int KS = taps * (CinP / 16);
    const size_t total = (size_t)ngroups * KS * 2 * 64 * 8;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
        const int e = (int)(idx & 7);
        const int lane = (int)((idx >> 3) & 63);
        const int nb = (int)((idx >> 9) & 1);
        const size_t rest = idx >> 10;
        const int ks = (int)(rest % KS), ng = (int)(rest / KS);
        const int tap = ks / (CinP / 16);
        const int c = (ks % (CinP / 16)) * 16 + (lane >> 5) * 8 + e;
        const int rho = lane & 31;
        const int o = ng * 64 + nb * 32 + ((rho >> 2) & 1) * 16 + (rho >> 3) * 4 + (rho & 3);
        T v = 0;
        if (c < Cin && o < Cout) v = w[weight_index(tap, c, o, taps, Cin, Cout, transposed)];
        packed[idx] = v;
    }
}

template <typename T>
__global__ void copy_weights(const T *__restrict__ w, T *__restrict__ packed, size_t total, int taps, int Cin, int Cout,
                             int transposed) {
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
        const int o = (int)(idx % Cout), c = (int)((idx / Cout) % Cin), tap = (int)(idx / ((size_t)Cout * Cin));
        packed[idx] = w[weight_index(tap, c, o, taps, Cin, Cout, transposed)];
    }
}

template <int DT, bool FUSED, int kMB>
__global__ __launch_bounds__(256) void conv_mfma(ConvParams p) {
    constexpr int PP = 64 * kMB;                // output pixels per pass
    extern __shared__ __align__(16) unsigned char lds[];
    const uint16_t *in = (const uint16_t *)p.in;
    uint16_t *out = (uint16_t *)p.out;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = lane >> 4, l16 = lane & 15;
    const int nact = min(*p.count, p.cap);
    const int M = p.oh * p.ow;
    const int pix_stride = (p.CC + 8) * 2;  // bytes between pixels in LDS
    const int c32_total = p.CinP / 32;
    const int KS = p.kh * p.kw * c32_total;
    const uint32_t per_tile = (uint32_t)p.mpasses * p.ngroups;
    const uint32_t items = (uint32_t)nact * per_tile;

    for (uint32_t item = blockIdx.x; item < items; item += gridDim.x) {
        const uint32_t b = fdiv(item, p.div_pn);
        const uint32_t rest = item - b * per_tile;
        const int pass = (int)fdiv(rest, p.div_ng);
        const int ng = (int)rest - pass * p.ngroups;

        int n = 0, y0 = 0, x0 = 0, oy0 = 0, ox0 = 0;
        if (FUSED) {
            n = p.indices[3 * b];
            const int by = p.indices[3 * b + 1], bx = p.indices[3 * b + 2];
            y0 = p.g_in.boffset_h + by * p.g_in.bstride_h;
            x0 = p.g_in.boffset_w + bx * p.g_in.bstride_w;
            oy0 = p.g_out.boffset_h + by * p.g_out.bstride_h;
            ox0 = p.g_out.boffset_w + bx * p.g_out.bstride_w;
        }

        // output pixels of this pass and the input rows they need
        const int p_lo = pass * PP, p_hi = min(p_lo + PP, M);
        const int i_lo = (int)fdiv(p_lo, p.div_ow), i_hi = (int)fdiv(p_hi - 1, p.div_ow);
        const int r_lo = i_lo * p.sh;
        const int nrows = (i_hi - i_lo) * p.sh + p.kh;

        // per-lane LDS byte offset of each of this wave's pixel blocks (tap (0,0), channel 0)
        int xbase[kMB];
        int pixel[kMB];
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb) {
            int px = p_lo + (wave * kMB + mb) * 16 + l16;
            pixel[mb] = px;
            px = min(px, M - 1);
            const int i = (int)fdiv(px, p.div_ow), j = px - i * p.ow;
            xbase[mb] = ((i * p.sh - r_lo) * p.tw + j * p.sw) * pix_stride + q * 16;
        }

        f32x4 acc[kMB][kNB];
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
            for (int nb = 0; nb < kNB; ++nb) acc[mb][nb] = (f32x4){0.f, 0.f, 0.f, 0.f};

        for (int chunk = 0; chunk < p.nchunks; ++chunk) {
            const int c0 = chunk * p.CC;
            const int cc = min(p.CC, p.CinP - c0);      // channels in this chunk (multiple of 32)
            const int cv = cc >> 3;                     // 16-byte vectors per pixel
            const FastDiv dcv = (chunk == p.nchunks - 1) ? p.div_cv_last : p.div_cv;
            __syncthreads();                            // previous chunk / item fully consumed
            const uint32_t nvec = (uint32_t)nrows * p.tw * cv;
            // kStage independent global loads in flight per thread before the LDS stores: a tile costs
            // nvec / (256 * kStage) memory round trips
            for (uint32_t v0 = threadIdx.x; v0 < nvec; v0 += 256 * kStage) {
                uint4 val[kStage];
                uint32_t dst[kStage];
#pragma unroll
                for (int u = 0; u < kStage; ++u) {
                    const uint32_t v = v0 + u * 256;
                    const uint32_t px = fdiv(v, dcv);
                    const int c8 = (int)(v - px * cv);
                    const int row = (int)fdiv(px, p.div_tw), col = (int)px - row * p.tw;
                    const int c = c0 + c8 * 8;
                    val[u] = make_uint4(0, 0, 0, 0);
                    dst[u] = px * pix_stride + c8 * 16;
                    if (v < nvec && c < p.Cin) {
                        if (FUSED) {
                            const int gy = y0 + r_lo + row, gx = x0 + col;
                            if (gy >= 0 && gy < p.H && gx >= 0 && gx < p.W)
                                val[u] = *(const uint4 *)(in + (((size_t)n * p.H + gy) * p.W + gx) * p.Cin + c);
                        } else {
                            val[u] = *(const uint4 *)(in + (((size_t)b * p.th + r_lo + row) * p.tw + col) * p.Cin + c);
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < kStage; ++u)
                    if (v0 + u * 256 < nvec) *(uint4 *)(lds + dst[u]) = val[u];
            }
            __syncthreads();

            // k loop over (tap row, tap column, 32-channel step).  The weight fragments come from L2 through a
            // ring of kWD steps: the fragments of step i + kWD are requested when step i has consumed its slot, so a
            // request has kWD steps of matrix work to land (one step is ~0.2 us, an L2 round trip several times
            // that).  The body of the main loop is kWD steps of straight-line code, which keeps the wait counts
            // exact; requests past the last step repeat it (harmless) instead of branching.
            const int steps = cc >> 5;
            const int nit = p.kh * p.kw * steps;
            const uint4 *wbase = (const uint4 *)p.w + ((size_t)ng * KS + (c0 >> 5)) * kNB * 64 + lane;
            int lt = 0, lst = 0;                       // request cursor: tap, channel step
            uint4 ring[kWD][kNB];
            auto request = [&](int slot) __attribute__((always_inline)) {
                const uint4 *wp = wbase + ((size_t)(lt * c32_total + lst) * kNB) * 64;
#pragma unroll
                for (int nb = 0; nb < kNB; ++nb) ring[slot][nb] = wp[(size_t)nb * 64];
                // advance, but never past the last step
                const bool last = (lt == p.kh * p.kw - 1) && (lst == steps - 1);
                if (!last) {
                    if (++lst == steps) { lst = 0; ++lt; }
                }
            };
            int r = 0, t = 0, st = 0;                  // use cursor: tap row, tap column, channel step
            auto one_step = [&](int slot) __attribute__((always_inline)) {
                const int off = (r * p.tw + t) * pix_stride + st * 64;
                uint4 xf[kMB];
#pragma unroll
                for (int mb = 0; mb < kMB; ++mb) xf[mb] = *(const uint4 *)(lds + xbase[mb] + off);
#pragma unroll
                for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
                    for (int nb = 0; nb < kNB; ++nb) acc[mb][nb] = mfma16x16x32<DT>(ring[slot][nb], xf[mb], acc[mb][nb]);
                if (++st == steps) { st = 0; if (++t == p.kw) { t = 0; ++r; } }
            };
#pragma unroll
            for (int u = 0; u < kWD; ++u) request(u);
            int it = 0;
            for (; it + kWD <= nit; it += kWD) {
#pragma unroll
                for (int u = 0; u < kWD; ++u) {
                    one_step(u);
                    request(u);
                }
            }
#pragma unroll
            for (int u = 0; u < kWD - 1; ++u)
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
            const int i = (int)fdiv(px, p.div_ow), j = px - i * p.ow;
            uint16_t *dst;
            if (FUSED) {
                const int gy = oy0 + i, gx = ox0 + j;
                if (gy < 0 || gy >= p.Ho || gx < 0 || gx >= p.Wo) continue;
                dst = out + (((size_t)n * p.Ho + gy) * p.Wo + gx) * p.Cout;
            } else {
                dst = out + ((size_t)b * M + px) * p.Cout;
            }
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int o0 = ng * 64 + half * 32 + q * 8;
                if (o0 >= p.Cout) continue;   // Cout % 8 == 0: a vector is all in or all out
                float v[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    float a = acc[mb][half * 2 + (k >> 2)][k & 3] + bias[half * 8 + k];
                    v[k] = p.relu ? fmaxf(a, 0.f) : a;
                }
                uint4 *d4 = (uint4 *)(dst + o0);
                if (FUSED && p.add) {
                    const uint4 old = *d4;
                    v[0] += unpack_lo<DT>(old.x); v[1] += unpack_hi<DT>(old.x);
                    v[2] += unpack_lo<DT>(old.y); v[3] += unpack_hi<DT>(old.y);
                    v[4] += unpack_lo<DT>(old.z); v[5] += unpack_hi<DT>(old.z);
                    v[6] += unpack_lo<DT>(old.w); v[7] += unpack_hi<DT>(old.w);
                }
                *d4 = make_uint4(pack2<DT>(v[0], v[1]), pack2<DT>(v[2], v[3]), pack2<DT>(v[4], v[5]), pack2<DT>(v[6], v[7]));
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
static bool use_mfma(sbnet_dtype dt, int Cin, int Cout) {
    return (dt == SBNET_BF16 || dt == SBNET_F16) && Cin % 8 == 0 && Cout % 8 == 0;
}

static size_t packed_elems(sbnet_dtype dt, int kh, int kw, int Cin, int Cout) {
    if (use_mfma(dt, Cin, Cout)) {
        const size_t CinP = ((size_t)Cin + 31) / 32 * 32, CoutP = ((size_t)Cout + 63) / 64 * 64;
        return 2 * (size_t)kh * kw * CinP * CoutP;      // 16x16x32 operand order, then 32x32x16 operand order
    }
    return (size_t)kh * kw * Cin * Cout;
}

static sbnet_status check_conv_shape(const char *who, sbnet_dtype dt, int cap, int th, int tw, int Cin, int kh,
                                     int kw, int sh, int sw, int Cout) {
    if (!is_float_dtype(dt)) return fail(SBNET_EUNSUPPORTED, "%s: dtype must be f32, bf16 or f16", who);
    if (cap < 0 || th <= 0 || tw <= 0 || Cin <= 0 || Cout <= 0 || kh <= 0 || kw <= 0 || sh <= 0 || sw <= 0)
        return fail(SBNET_EINVAL, "%s: bad sizes", who);
    if (kh > th || kw > tw) return fail(SBNET_EINVAL, "%s: kernel larger than tile", who);
    return SBNET_OK;
}

static const int kLdsBudget = 64 * 1024;      // preferred: two workgroups per CU
static const int kLdsMax = 160 * 1024;        // gfx950 LDS per workgroup

template <bool FUSED>
static sbnet_status run_conv(const char *who, sbnet_dtype dt, ConvParams &p, hipStream_t s) {
    if (p.cap == 0) return SBNET_OK;
    p.oh = (p.th - p.kh) / p.sh + 1;
    p.ow = (p.tw - p.kw) / p.sw + 1;
    const long long M = (long long)p.oh * p.ow;
    if (M * p.Cout >= (1LL << 31) || (long long)p.th * p.tw * p.Cin >= (1LL << 31))
        return fail(SBNET_EUNSUPPORTED, "%s: tile too large", who);
    p.div_ow = make_fastdiv(p.ow);
    p.div_tw = make_fastdiv(p.tw);

    if (use_mfma(dt, p.Cin, p.Cout)) p.w32_offset = packed_elems(dt, p.kh, p.kw, p.Cin, p.Cout) / 2 / 8;
    sbnet_status st16 = SBNET_OK;
    if (conv16_try(dt, FUSED, p, s, &st16, who)) return st16;
    if (conv3_try(dt, FUSED, p, s, &st16, who)) return st16;

    if (!use_mfma(dt, p.Cin, p.Cout)) {
        p.div_cv = make_fastdiv(p.Cout);
        const long long per_tile = M * p.Cout;
        dim3 grid((unsigned)((per_tile + 255) / 256 > 64 ? 64 : (per_tile + 255) / 256), (unsigned)(p.cap > 4096 ? 4096 : p.cap));
#define SBNET_DIRECT(DT) hipLaunchKernelGGL((conv_direct<DT, FUSED>), grid, dim3(256), 0, s, p)
        if (dt == SBNET_F32) SBNET_DIRECT(SBNET_F32);
        else if (dt == SBNET_BF16) SBNET_DIRECT(SBNET_BF16);
        else SBNET_DIRECT(SBNET_F16);
#undef SBNET_DIRECT
        return launch_status(who);
    }

    p.CinP = (p.Cin + 31) / 32 * 32;
    p.ngroups = (p.Cout + 63) / 64;
    // pixels per pass: 256, or 64 when even the caller's bound on the active blocks gives fewer work items than CUs
    const int PP = ((long long)p.cap * ((M + 255) / 256) * p.ngroups < 256) ? 64 : 256;
    p.mpasses = (int)((M + PP - 1) / PP);
    // rows of input a pass of PP consecutive output pixels can touch
    int out_rows = (PP + p.ow - 1) / p.ow + ((PP % p.ow) ? 1 : 0);
    if (out_rows > p.oh) out_rows = p.oh;
    int lds_rows = (out_rows - 1) * p.sh + p.kh;
    if (lds_rows > p.th) lds_rows = p.th;
    p.lds_rows = lds_rows;
    const long long px = (long long)lds_rows * p.tw;
    int CC = p.CinP;
    while (CC > 32 && px * (CC + 8) * 2 > kLdsBudget) CC -= 32;
    const long long lds_bytes = px * (CC + 8) * 2;
    if (lds_bytes > kLdsMax) return fail(SBNET_EUNSUPPORTED, "%s: tile rows do not fit in LDS", who);
    p.CC = CC;
    p.nchunks = (p.CinP + CC - 1) / CC;
    p.div_cv = make_fastdiv(CC / 8);
    p.div_cv_last = make_fastdiv((p.CinP - (p.nchunks - 1) * CC) / 8);
    p.div_pn = make_fastdiv((uint32_t)p.mpasses * p.ngroups);
    p.div_ng = make_fastdiv(p.ngroups);
    const long long items = (long long)p.cap * p.mpasses * p.ngroups;
    if (items >= (1LL << 31)) return fail(SBNET_EUNSUPPORTED, "%s: too many work items", who);
    const int grid = (int)(items < 8192 ? items : 8192);

#define SBNET_MFMA(DT, MB)                                                                                     \
    do {                                                                                                       \
        if (lds_bytes > 48 * 1024)                                                                             \
            (void)hipFuncSetAttribute((const void *)conv_mfma<DT, FUSED, MB>,                                  \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);             \
        hipLaunchKernelGGL((conv_mfma<DT, FUSED, MB>), dim3(grid), dim3(256), (size_t)lds_bytes, s, p);        \
    } while (0)
    if (dt == SBNET_BF16) {
        if (PP == 256) SBNET_MFMA(SBNET_BF16, 4);
        else SBNET_MFMA(SBNET_BF16, 1);
    } else {
        if (PP == 256) SBNET_MFMA(SBNET_F16, 4);
        else SBNET_MFMA(SBNET_F16, 1);
    }
#undef SBNET_MFMA
    return launch_status(who);
}

}  // namespace sbnet

using namespace sbnet;

// Cin, Cout: of the convolution the packed weights serve (for the transposed form: the forward convolution's Cout, Cin)
static sbnet_status pack_entry(const char *who, const void *w_hwio, sbnet_dtype dtype, int kh, int kw, int Cin, int Cout,
                               void *w_packed, size_t *bytes, int transposed, void *stream) {
    if (!is_float_dtype(dtype)) return fail(SBNET_EUNSUPPORTED, "%s: dtype must be f32, bf16 or f16", who);
    if (kh <= 0 || kw <= 0 || Cin <= 0 || Cout <= 0) return fail(SBNET_EINVAL, "%s: bad sizes", who);
    const size_t elems = packed_elems(dtype, kh, kw, Cin, Cout);
    if (bytes) *bytes = elems * elem_bytes(dtype);
    if (!w_packed) {
        if (!bytes) return fail(SBNET_EINVAL, "%s: nothing to do", who);
        return SBNET_OK;
    }
    if (!w_hwio) return fail(SBNET_EINVAL, "%s: null weights", who);
    hipStream_t s = (hipStream_t)stream;
    const int grid = (int)((elems + 255) / 256 < 4096 ? (elems + 255) / 256 : 4096);
    if (use_mfma(dtype, Cin, Cout)) {
        const int CinP = (Cin + 31) / 32 * 32, ngroups = (Cout + 63) / 64;
        hipLaunchKernelGGL(pack_mfma_weights<uint16_t>, dim3(grid), dim3(256), 0, s, (const uint16_t *)w_hwio,
                           (uint16_t *)w_packed, kh * kw, Cin, Cout, CinP, ngroups, transposed);
        hipLaunchKernelGGL(pack_mfma32_weights<uint16_t>, dim3(grid), dim3(256), 0, s, (const uint16_t *)w_hwio,
                           (uint16_t *)w_packed + elems / 2, kh * kw, Cin, Cout, CinP, ngroups, transposed);
    } else if (dtype == SBNET_F32) {
        hipLaunchKernelGGL(copy_weights<uint32_t>, dim3(grid), dim3(256), 0, s, (const uint32_t *)w_hwio,
                           (uint32_t *)w_packed, elems, kh * kw, Cin, Cout, transposed);
    } else {
        hipLaunchKernelGGL(copy_weights<uint16_t>, dim3(grid), dim3(256), 0, s, (const uint16_t *)w_hwio,
                           (uint16_t *)w_packed, elems, kh * kw, Cin, Cout, transposed);
    }
    return launch_status(who);
}

extern "C" sbnet_status sbnet_pack_weights(const void *w_hwio, sbnet_dtype dtype, int kh, int kw, int Cin, int Cout,
                                           void *w_packed, size_t *bytes, void *stream) {
    return pack_entry("sbnet_pack_weights", w_hwio, dtype, kh, kw, Cin, Cout, w_packed, bytes, 0, stream);
}

extern "C" sbnet_status sbnet_pack_weights_transposed(const void *w_hwio, sbnet_dtype dtype, int kh, int kw, int Cin,
                                                      int Cout, void *w_packed, size_t *bytes, void *stream) {
    return pack_entry("sbnet_pack_weights_transposed", w_hwio, dtype, kh, kw, Cout, Cin, w_packed, bytes, 1, stream);
}

extern "C" sbnet_status sbnet_conv_on_tiles(const void *tiles_in, sbnet_dtype dtype, const int32_t *count, int cap,
                                            int th, int tw, int Cin, const void *w_packed, const float *bias, int kh,
                                            int kw, int sh, int sw, int Cout, int relu, void *tiles_out,
                                            void *stream) {
    const char *who = "sbnet_conv_on_tiles";
    if (!tiles_in || !count || !w_packed || !tiles_out) return fail(SBNET_EINVAL, "%s: null pointer", who);
    sbnet_status st = check_conv_shape(who, dtype, cap, th, tw, Cin, kh, kw, sh, sw, Cout);
    if (st != SBNET_OK) return st;
    if (((uintptr_t)tiles_in | (uintptr_t)tiles_out | (uintptr_t)w_packed) & 15)
        return fail(SBNET_EINVAL, "%s: pointers must be 16-byte aligned", who);
    ConvParams p = {};
    p.in = tiles_in; p.out = tiles_out; p.w = w_packed; p.bias = bias;
    p.count = count; p.cap = cap;
    p.th = th; p.tw = tw; p.Cin = Cin; p.Cout = Cout;
    p.kh = kh; p.kw = kw; p.sh = sh; p.sw = sw; p.relu = relu ? 1 : 0;
    return run_conv<false>(who, dtype, p, (hipStream_t)stream);
}

// ---- data gradient of the tile convolution ----------------------------------------------------------------------
// The gradient of a strided valid convolution with respect to its input is itself a stride-1 valid convolution: of
// the output gradient spread out by the stride (zeros between its pixels) and framed by kh-1 / kw-1 zeros, with the
// taps mirrored and the channel roles exchanged.  At stride 1 the fused kernels read that frame for free (a tile of
// the output gradient is addressed as a small image, whose surroundings read as zeros); at larger strides
// spread_tiles builds the framed stack.  The convolution kernels of this file then do the arithmetic with weights
// packed by sbnet_pack_weights_transposed.
namespace sbnet {

template <typename V>
__global__ void spread_tiles(const V *__restrict__ dout, V *__restrict__ framed, const int32_t *__restrict__ count,
                             int cap, int oh, int ow, int ph, int pw, int cv, int kh, int kw, int sh, int sw,
                             FastDiv div_cv, FastDiv div_pw) {
    int n = *count;
    if (n > cap) n = cap;
    const uint32_t per_tile = (uint32_t)ph * pw * cv;
    for (int b = blockIdx.y; b < n; b += gridDim.y) {
        for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < per_tile; i += gridDim.x * blockDim.x) {
            const uint32_t px = fdiv(i, div_cv), c = i - px * cv;
            const uint32_t y = fdiv(px, div_pw), x = px - y * pw;
            const int u = (int)y - (kh - 1), v = (int)x - (kw - 1);
            V val = {};
            if (u >= 0 && v >= 0 && u % sh == 0 && v % sw == 0 && u / sh < oh && v / sw < ow)
                val = dout[(((size_t)b * oh + u / sh) * ow + v / sw) * cv + c];
            framed[(size_t)b * per_tile + i] = val;
        }
    }
}

// index triple (b, 0, 0) for tile b: every tile as a sample of its own with a single block
__global__ void tile_indices(int32_t *__restrict__ idx, int cap) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < cap) {
        idx[3 * b] = b;
        idx[3 * b + 1] = 0;
        idx[3 * b + 2] = 0;
    }
}

}  // namespace sbnet

static size_t framed_elems(int cap, int th, int tw, int kh, int kw, int Cout) {
    return (size_t)cap * (size_t)(th + kh - 1) * (size_t)(tw + kw - 1) * (size_t)Cout;
}

extern "C" size_t sbnet_conv_backward_data_workspace_bytes(sbnet_dtype dtype, int cap, int th, int tw, int kh, int kw,
                                                           int sh, int sw, int Cout) {
    if (!is_float_dtype(dtype) || cap < 0 || th <= 0 || tw <= 0 || kh <= 0 || kw <= 0 || sh <= 0 || sw <= 0 || Cout <= 0)
        return 0;
    // stride 1: one index triple per tile; otherwise the framed copy of the output gradient
    const size_t bytes = (sh == 1 && sw == 1) ? (size_t)cap * 12 : framed_elems(cap, th, tw, kh, kw, Cout) * elem_bytes(dtype);
    return (bytes + 255) / 256 * 256;
}

extern "C" sbnet_status sbnet_conv_on_tiles_backward_data(const void *dout_tiles, sbnet_dtype dtype,
                                                          const int32_t *count, int cap, int th, int tw, int Cin,
                                                          const void *w_packed_t, int kh, int kw, int sh, int sw,
                                                          int Cout, void *din_tiles, void *workspace,
                                                          size_t workspace_bytes, void *stream) {
    const char *who = "sbnet_conv_on_tiles_backward_data";
    if (!dout_tiles || !count || !w_packed_t || !din_tiles || !workspace)
        return fail(SBNET_EINVAL, "%s: null pointer", who);
    sbnet_status st = check_conv_shape(who, dtype, cap, th, tw, Cin, kh, kw, sh, sw, Cout);
    if (st != SBNET_OK) return st;
    if (((uintptr_t)dout_tiles | (uintptr_t)din_tiles | (uintptr_t)w_packed_t | (uintptr_t)workspace) & 15)
        return fail(SBNET_EINVAL, "%s: pointers must be 16-byte aligned", who);
    if (workspace_bytes < sbnet_conv_backward_data_workspace_bytes(dtype, cap, th, tw, kh, kw, sh, sw, Cout))
        return fail(SBNET_EINVAL, "%s: workspace too small", who);
    if (cap == 0) return SBNET_OK;
    const int oh = (th - kh) / sh + 1, ow = (tw - kw) / sw + 1;
    const int ph = th + kh - 1, pw = tw + kw - 1;
    const size_t row_bytes = (size_t)Cout * elem_bytes(dtype);
    if ((long long)ph * pw * (long long)row_bytes >= (1LL << 31))
        return fail(SBNET_EUNSUPPORTED, "%s: tile too large", who);
    hipStream_t s = (hipStream_t)stream;
    if (sh == 1 && sw == 1 && kh == 1 && kw == 1) {
        // A pointwise convolution has no frame either: its data gradient is the pointwise convolution of the tiles of
        // dout with the exchanged weights, tile for tile.
        ConvParams p = {};
        p.in = dout_tiles; p.out = din_tiles; p.w = w_packed_t; p.bias = nullptr;
        p.count = count; p.cap = cap;
        p.th = th; p.tw = tw; p.Cin = Cout; p.Cout = Cin;
        p.kh = 1; p.kw = 1; p.sh = 1; p.sw = 1; p.relu = 0;
        return run_conv<false>(who, dtype, p, s);
    }
    if (sh == 1 && sw == 1) {
        // No stride, nothing to spread: the frame of zeros is what the fused kernels read around an image anyway.
        // Every tile of dout is taken as a sample of its own (oh x ow), gathered with a window that starts kh-1 / kw-1
        // outside it, and the result "scattered" into a th x tw image that is the tile of din.
        int32_t *idx = (int32_t *)workspace;
        hipLaunchKernelGGL(tile_indices, dim3((cap + 255) / 256), dim3(256), 0, s, idx, cap);
        st = launch_status(who);
        if (st != SBNET_OK) return st;
        ConvParams p = {};
        p.in = dout_tiles; p.out = din_tiles; p.w = w_packed_t; p.bias = nullptr;
        p.indices = idx; p.count = count; p.cap = cap;
        p.th = ph; p.tw = pw; p.Cin = Cout; p.Cout = Cin;
        p.kh = kh; p.kw = kw; p.sh = 1; p.sw = 1; p.relu = 0; p.add = 0;
        p.g_in.bsize_h = ph; p.g_in.bsize_w = pw; p.g_in.bstride_h = ph; p.g_in.bstride_w = pw;
        p.g_in.boffset_h = -(kh - 1); p.g_in.boffset_w = -(kw - 1); p.g_in.bcount_h = p.g_in.bcount_w = 1;
        p.g_out.bsize_h = th; p.g_out.bsize_w = tw; p.g_out.bstride_h = th; p.g_out.bstride_w = tw;
        p.g_out.boffset_h = p.g_out.boffset_w = 0; p.g_out.bcount_h = p.g_out.bcount_w = 1;
        p.H = oh; p.W = ow; p.Ho = th; p.Wo = tw;
        return run_conv<true>(who, dtype, p, s);
    }
    const int vb = row_bytes % 16 == 0 ? 16 : row_bytes % 8 == 0 ? 8 : row_bytes % 4 == 0 ? 4 : 2;
    const int cv = (int)(row_bytes / vb);
    const long long per_tile = (long long)ph * pw * cv;
    dim3 grid((unsigned)((per_tile + 255) / 256 > 64 ? 64 : (per_tile + 255) / 256),
              (unsigned)(cap > 4096 ? 4096 : cap));
#define SBNET_SPREAD(V)                                                                                          \
    hipLaunchKernelGGL((spread_tiles<V>), grid, dim3(256), 0, s, (const V *)dout_tiles, (V *)workspace, count,  \
                       cap, oh, ow, ph, pw, cv, kh, kw, sh, sw, make_fastdiv(cv), make_fastdiv(pw))
    if (vb == 16) SBNET_SPREAD(uint4);
    else if (vb == 8) SBNET_SPREAD(uint2);
    else if (vb == 4) SBNET_SPREAD(uint32_t);
    else SBNET_SPREAD(uint16_t);
#undef SBNET_SPREAD
    st = launch_status(who);
    if (st != SBNET_OK) return st;
    // the gradient as a stride-1 convolution of the framed stack: Cout channels in, Cin channels out
    ConvParams p = {};
    p.in = workspace; p.out = din_tiles; p.w = w_packed_t; p.bias = nullptr;
    p.count = count; p.cap = cap;
    p.th = ph; p.tw = pw; p.Cin = Cout; p.Cout = Cin;
    p.kh = kh; p.kw = kw; p.sh = 1; p.sw = 1; p.relu = 0;
    return run_conv<false>(who, dtype, p, s);
}

extern "C" sbnet_status sbnet_sparse_conv(const void *x, sbnet_dtype dtype, int N, int H, int W, int Cin,
                                          const int32_t *indices, const int32_t *count, int cap,
                                          const sbnet_geom *g_in, const sbnet_geom *g_out, const void *w_packed,
                                          const float *bias, int kh, int kw, int sh, int sw, int Cout, int relu,
                                          void *y, int H_out, int W_out, int add, void *stream) {
    const char *who = "sbnet_sparse_conv";
    if (!x || !indices || !count || !w_packed || !y) return fail(SBNET_EINVAL, "%s: null pointer", who);
    if (N <= 0 || H <= 0 || W <= 0 || H_out <= 0 || W_out <= 0) return fail(SBNET_EINVAL, "%s: bad sizes", who);
    if (!geom_ok(g_in) || !geom_ok(g_out)) return fail(SBNET_EINVAL, "%s: bad geometry", who);
    sbnet_status st = check_conv_shape(who, dtype, cap, g_in->bsize_h, g_in->bsize_w, Cin, kh, kw, sh, sw, Cout);
    if (st != SBNET_OK) return st;
    if ((g_in->bsize_h - kh) / sh + 1 != g_out->bsize_h || (g_in->bsize_w - kw) / sw + 1 != g_out->bsize_w)
        return fail(SBNET_EINVAL, "%s: output block does not match the convolution of the input tile", who);
    if (g_out->bstride_h < g_out->bsize_h || g_out->bstride_w < g_out->bsize_w)
        return fail(SBNET_EINVAL, "%s: output blocks must not overlap", who);
    if (ranges_overlap(x, (size_t)N * H * W * Cin * elem_bytes(dtype), y, (size_t)N * H_out * W_out * Cout * elem_bytes(dtype)))
        return fail(SBNET_EINVAL, "%s: y must not overlap x", who);
    if (((uintptr_t)x | (uintptr_t)y | (uintptr_t)w_packed) & 15)
        return fail(SBNET_EINVAL, "%s: pointers must be 16-byte aligned", who);
    ConvParams p = {};
    p.in = x; p.out = y; p.w = w_packed; p.bias = bias;
    p.indices = indices; p.count = count; p.cap = cap;
    p.th = g_in->bsize_h; p.tw = g_in->bsize_w; p.Cin = Cin; p.Cout = Cout;
    p.kh = kh; p.kw = kw; p.sh = sh; p.sw = sw; p.relu = relu ? 1 : 0; p.add = add ? 1 : 0;
    p.g_in = *g_in; p.g_out = *g_out;
    p.H = H; p.W = W; p.Ho = H_out; p.Wo = W_out;
    return run_conv<true>(who, dtype, p, (hipStream_t)stream);
}

// Block flags in, convolved active blocks out: the fused convolution with reduce_mask's compaction folded into its
// prologue where the kernel can take flags (3x3 stride 1, 16 x 16 output blocks, 32 or 64 input channels, bf16 / f16);
// other shapes compact the flags in a launch of their own and run sbnet_sparse_conv.  Either way indices / count hold
// the list afterwards.
extern "C" sbnet_status sbnet_sparse_conv_from_flags(const uint8_t *flags, const void *x, sbnet_dtype dtype, int N, int H,
                                                     int W, int Cin, int32_t *indices, int32_t *count, int cap,
                                                     const sbnet_geom *g_in, const sbnet_geom *g_out, const void *w_packed,
                                                     const float *bias, int kh, int kw, int sh, int sw, int Cout, int relu,
                                                     void *y, int H_out, int W_out, int add, void *stream) {
    const char *who = "sbnet_sparse_conv_from_flags";
    if (!flags || !x || !indices || !count || !w_packed || !y) return fail(SBNET_EINVAL, "%s: null pointer", who);
    if (N <= 0 || H <= 0 || W <= 0 || H_out <= 0 || W_out <= 0 || cap < 0) return fail(SBNET_EINVAL, "%s: bad sizes", who);
    if (!geom_ok(g_in) || !geom_ok(g_out)) return fail(SBNET_EINVAL, "%s: bad geometry", who);
    if (g_out->bcount_h != g_in->bcount_h || g_out->bcount_w != g_in->bcount_w)
        return fail(SBNET_EINVAL, "%s: g_in and g_out must describe one block grid", who);
    if (!mask_flag_path(N, g_in)) return fail(SBNET_EUNSUPPORTED, "%s: more blocks than the flag form takes", who);
    if (((uintptr_t)flags) & 15) return fail(SBNET_EINVAL, "%s: flags must be 16-byte aligned", who);
    hipStream_t s = (hipStream_t)stream;
    bool fold = cap > 0 && is_float_dtype(dtype) &&
                !ranges_overlap(x, (size_t)N * H * W * Cin * elem_bytes(dtype), y, (size_t)N * H_out * W_out * Cout * elem_bytes(dtype)) &&
                !(((uintptr_t)x | (uintptr_t)y | (uintptr_t)w_packed) & 15) &&
                check_conv_shape(who, dtype, cap, g_in->bsize_h, g_in->bsize_w, Cin, kh, kw, sh, sw, Cout) == SBNET_OK &&
                (g_in->bsize_h - kh) / sh + 1 == g_out->bsize_h && (g_in->bsize_w - kw) / sw + 1 == g_out->bsize_w &&
                g_out->bstride_h >= g_out->bsize_h && g_out->bstride_w >= g_out->bsize_w && use_mfma(dtype, Cin, Cout);
    ConvParams p = {};
    if (fold) {
        p.in = x; p.out = y; p.w = w_packed; p.bias = bias;
        p.cap = cap;
        p.th = g_in->bsize_h; p.tw = g_in->bsize_w; p.Cin = Cin; p.Cout = Cout;
        p.kh = kh; p.kw = kw; p.sh = sh; p.sw = sw; p.relu = relu ? 1 : 0; p.add = add ? 1 : 0;
        p.g_in = *g_in; p.g_out = *g_out;
        p.H = H; p.W = W; p.Ho = H_out; p.Wo = W_out;
        p.oh = g_out->bsize_h; p.ow = g_out->bsize_w;
        p.w32_offset = packed_elems(dtype, kh, kw, Cin, Cout) / 2 / 8;
        p.flags = flags;
        p.total_blocks = N * g_in->bcount_h * g_in->bcount_w;
        p.indices_out = indices; p.count_out = count;
        fold = conv16_accepts(dtype, true, p);
    }
    if (!fold) {
        sbnet_status st = flags_to_indices(who, flags, N, g_in, indices, count, cap, s);
        if (st != SBNET_OK) return st;
        return sbnet_sparse_conv(x, dtype, N, H, W, Cin, indices, count, cap, g_in, g_out, w_packed, bias, kh, kw, sh, sw, Cout,
                                 relu, y, H_out, W_out, add, stream);
    }
    sbnet_status st = SBNET_OK;
    if (!conv16_try(dtype, true, p, s, &st, who)) return fail(SBNET_EHIP, "%s: internal dispatch error", who);
    return st;
}

// Mask in, convolved active blocks out, in one call: sbnet_block_flags + sbnet_sparse_conv_from_flags where the grid is
// small enough for flags, sbnet_reduce_mask + sbnet_sparse_conv beyond.
extern "C" sbnet_status sbnet_sparse_conv_from_mask(const void *mask, sbnet_dtype mask_dtype, int mask_H, int mask_W,
                                                    const sbnet_geom *g_mask, sbnet_pool pool, float threshold,
                                                    const void *x, sbnet_dtype dtype, int N, int H, int W, int Cin,
                                                    int32_t *indices, int32_t *count, int cap, const sbnet_geom *g_in,
                                                    const sbnet_geom *g_out, const void *w_packed, const float *bias,
                                                    int kh, int kw, int sh, int sw, int Cout, int relu, void *y, int H_out,
                                                    int W_out, int add, void *workspace, size_t workspace_bytes,
                                                    void *stream) {
    const char *who = "sbnet_sparse_conv_from_mask";
    if (!mask || !workspace || !indices || !count) return fail(SBNET_EINVAL, "%s: null pointer", who);
    if (N <= 0 || !geom_ok(g_mask) || !geom_ok(g_in)) return fail(SBNET_EINVAL, "%s: bad sizes or geometry", who);
    if (g_mask->bcount_h != g_in->bcount_h || g_mask->bcount_w != g_in->bcount_w)
        return fail(SBNET_EINVAL, "%s: the geometries must describe one block grid", who);
    if (workspace_bytes < sbnet_workspace_bytes(N, g_mask)) return fail(SBNET_EINVAL, "%s: workspace too small", who);
    sbnet_status st;
    if (mask_flag_path(N, g_mask)) {
        st = sbnet_block_flags(mask, mask_dtype, N, mask_H, mask_W, g_mask, pool, threshold, (uint8_t *)workspace,
                               workspace_bytes, stream);
        if (st != SBNET_OK) return st;
        return sbnet_sparse_conv_from_flags((const uint8_t *)workspace, x, dtype, N, H, W, Cin, indices, count, cap, g_in, g_out,
                                            w_packed, bias, kh, kw, sh, sw, Cout, relu, y, H_out, W_out, add, stream);
    }
    st = sbnet_reduce_mask(mask, mask_dtype, N, mask_H, mask_W, g_mask, pool, threshold, indices, count, cap, workspace,
                           workspace_bytes, stream);
    if (st != SBNET_OK) return st;
    return sbnet_sparse_conv(x, dtype, N, H, W, Cin, indices, count, cap, g_in, g_out, w_packed, bias, kh, kw, sh, sw, Cout, relu,
                             y, H_out, W_out, add, stream);
}
