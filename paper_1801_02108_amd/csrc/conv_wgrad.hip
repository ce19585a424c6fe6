// Weight gradient of the tile convolution (training support for the convolution of Sec. 3.2 of arXiv 1801.02108):
//   dw[r][t][c][o] = sum over tiles b and output pixels (i, j) of x[b][r + sh i][t + sw j][c] * dout[b][i][j][o].
// The contraction runs over pixels, the one index that the channel-last tiles do not keep contiguous, and its result
// is small (kh kw Cin Cout numbers) while its inputs are the whole tile stacks.  So the tiles are split over many
// workgroups, each of which keeps a partial dw in registers for all its tiles and writes it once; a second kernel adds
// the partial results in a fixed order (no atomics: the result does not depend on scheduling).
//
// wgrad_mfma (3x3, stride 1 or 2, BF16/F16, channel counts multiples of 8): a workgroup owns 64 input by 64 output
// channels, one 32x32 block per wave with nine fp32 accumulators (one per tap).  Tiles pass through LDS a few output
// rows at a time (a "stage"), stored channel-major so that a lane's matrix operand (8 consecutive pixels of one
// channel) is one aligned 16-byte read:
//   * x rows are split by column phase (column % stride), so that the pixels a tap reads for consecutive output
//     pixels are consecutive; a tap's window starts 0 or 1 elements (stride 2) or 0, 1, 2 elements (stride 1) into a
//     16-byte vector and is cut from two neighbouring vectors with one byte-align per word;
//   * the channel planes are an odd number of 16-byte vectors apart and the vector index inside a plane is XOR-ed with
//     a function of the channel group: the 16-bit transposing writes of a wave (8 channel groups x 8 pixels) and the
//     16-byte operand reads (32 consecutive channels) both spread over all banks;
//   * columns beyond the output row and rows beyond the tile hold zeros, in both operands, so that a partial row or
//     stage adds nothing.
// Stages alternate between two LDS buffers: the loads of the next stage are issued before the matrix work of the
// current one and written to the other buffer after it.
//
// wgrad_direct: every other shape and fp32; one thread per weight, plain loops.
#include <hip/hip_runtime.h>

#include "conv_common.h"

namespace sbnet {
namespace {

struct WgradParams {
    const void *x;            // [cap][th][tw][Cin]
    const void *g;            // [cap][oh][ow][Cout]
    float *part;              // [nsplit][taps][CinP][CoutP]
    const int32_t *count;
    int cap, th, tw, oh, ow, Cin, Cout, kh, kw, sh, sw;
    int nsplit, ncb, nob, CinP, CoutP;
    uint32_t x_tile_bytes, g_tile_bytes;
};

template <int S, int NSEG>
struct WgradShape {
    static constexpr int R = 8 / (S * NSEG);              // output rows per stage
    static constexpr int RX = (R - 1) * S + 3;            // input rows per stage
    static constexpr int CPV = 2 * NSEG + 1;              // 16-byte vectors per phase row of x (one spare for the window)
    static constexpr int XPL = (RX * S * CPV + 7) / 8 * 8;
    static constexpr int CSX = XPL + 1;                   // vectors between channel planes of x (odd)
    static constexpr int GV = 2 * NSEG;                   // vectors per row of dout
    static constexpr int GPL = (R * GV + 7) / 8 * 8;
    static constexpr int CSG = GPL + 1;
    static constexpr int XBYTES = 64 * CSX * 16;
    static constexpr int STAGE = 64 * (CSX + CSG) * 16;
    static constexpr int TWMAX = 16 * NSEG * S + 2;
    static constexpr int NVX = (RX * TWMAX * 8 + 255) / 256;
    static constexpr int NVG = (R * 16 * NSEG * 8 + 255) / 256;
};

__device__ __forceinline__ uint4 lds_read16(const char *p) { return *(const uint4 *)p; }

// elements 1..8 of the 16 elements in (v0, v1)
__device__ __forceinline__ uint4 window1(uint4 v0, uint4 v1) {
    return make_uint4(__builtin_amdgcn_alignbyte(v0.y, v0.x, 2), __builtin_amdgcn_alignbyte(v0.z, v0.y, 2),
                      __builtin_amdgcn_alignbyte(v0.w, v0.z, 2), __builtin_amdgcn_alignbyte(v1.x, v0.w, 2));
}
// elements 2..9
__device__ __forceinline__ uint4 window2(uint4 v0, uint4 v1) { return make_uint4(v0.y, v0.z, v0.w, v1.x); }

// the 8 elements of a staged vector go to 8 consecutive channel planes (plane_bytes apart)
template <int PLANE_BYTES>
__device__ __forceinline__ void lds_write_transposed(char *p, uint4 d) {
    const uint32_t w[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        *(uint16_t *)(p + (2 * k) * PLANE_BYTES) = (uint16_t)(w[k] & 0xffffu);
        *(uint16_t *)(p + (2 * k + 1) * PLANE_BYTES) = (uint16_t)(w[k] >> 16);
    }
}

template <int DT, int S, int NSEG>
__global__ __launch_bounds__(256) void wgrad_mfma(WgradParams p) {
    typedef WgradShape<S, NSEG> Sh;
    constexpr int R = Sh::R, RX = Sh::RX, CPV = Sh::CPV, CSX = Sh::CSX, CSG = Sh::CSG, GV = Sh::GV;
    constexpr int NVX = Sh::NVX, NVG = Sh::NVG;
    extern __shared__ __align__(16) char lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sigma = blockIdx.x % p.nsplit, cbob = blockIdx.x / p.nsplit;
    const int cb = cbob / p.nob, ob = cbob - cb * p.nob;
    int n = *p.count;
    if (n > p.cap) n = p.cap;
    if (sigma >= n) return;                                        // the sum below reads no partial result of this split
    const int ntiles = (n - sigma + p.nsplit - 1) / p.nsplit;
    const int H = (p.oh + R - 1) / R;
    const int nstages = ntiles * H;

    // ---- what this thread stages: NVX vectors of x and NVG of dout per stage, fixed for the whole kernel ----------
    uint32_t relx[NVX], ldsx[NVX], relg[NVG], ldsg[NVG];
    const int cv = tid & 7;                                        // 8-channel group inside the workgroup's 64
    const uint32_t swz = 2u * (cv & 3);
#pragma unroll
    for (int u = 0; u < NVX; ++u) {
        const int px = (u * 256 + tid) >> 3;
        const int ry = px / p.tw, x = px - ry * p.tw;
        const int xs = x / S, ph = x - xs * S;
        const bool ok = ry < RX && cb * 64 + cv * 8 < p.Cin && xs < CPV * 8;
        relx[u] = ok ? (uint32_t)(((ry * p.tw + x) * p.Cin + cb * 64 + cv * 8) * 2) : kOutOfRange;
        const uint32_t v = (uint32_t)((ry * S + ph) * CPV + (xs >> 3)) ^ swz;
        ldsx[u] = (uint32_t)(cv * 8 * CSX * 16) + v * 16 + (xs & 7) * 2;
    }
#pragma unroll
    for (int u = 0; u < NVG; ++u) {
        const int px = (u * 256 + tid) >> 3;
        const int gy = px / p.ow, x = px - gy * p.ow;
        const bool ok = gy < R && ob * 64 + cv * 8 < p.Cout;
        relg[u] = ok ? (uint32_t)(((gy * p.ow + x) * p.Cout + ob * 64 + cv * 8) * 2) : kOutOfRange;
        const uint32_t v = (uint32_t)(gy * GV + (x >> 3)) ^ swz;
        ldsg[u] = (uint32_t)(Sh::XBYTES + cv * 8 * CSG * 16) + v * 16 + (x & 7) * 2;
    }
    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.x), 0, (int)((uint32_t)p.cap * p.x_tile_bytes), kBufWord3);
    const __amdgpu_buffer_rsrc_t gr = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.g), 0, (int)((uint32_t)p.cap * p.g_tile_bytes), kBufWord3);
    const uint32_t x_stage_step = (uint32_t)(R * S * p.tw * p.Cin * 2), g_stage_step = (uint32_t)(R * p.ow * p.Cout * 2);

    uint4 xv[NVX], gv[NVG];
    auto issue = [&](int b, int h) {
        const uint32_t x0 = (uint32_t)h * x_stage_step, g0 = (uint32_t)h * g_stage_step;
#pragma unroll
        for (int u = 0; u < NVX; ++u) {
            const uint32_t o = x0 + relx[u];                       // rows beyond the tile: zeros
            xv[u] = buf_load16(xr, o < p.x_tile_bytes ? (uint32_t)b * p.x_tile_bytes + o : kOutOfRange);
        }
#pragma unroll
        for (int u = 0; u < NVG; ++u) {
            const uint32_t o = g0 + relg[u];
            gv[u] = buf_load16(gr, o < p.g_tile_bytes ? (uint32_t)b * p.g_tile_bytes + o : kOutOfRange);
        }
    };
    auto write = [&](int bufno) {
        char *base = lds + bufno * Sh::STAGE;
#pragma unroll
        for (int u = 0; u < NVX; ++u)
            if (relx[u] != kOutOfRange) lds_write_transposed<CSX * 16>(base + ldsx[u], xv[u]);
#pragma unroll
        for (int u = 0; u < NVG; ++u)
            if (relg[u] != kOutOfRange) lds_write_transposed<CSG * 16>(base + ldsg[u], gv[u]);
    };

    // ---- matrix operands of this wave ------------------------------------------------------------------------------
    const int cl = (wave >> 1) * 32 + (lane & 31), ol = (wave & 1) * 32 + (lane & 31), m = lane >> 5;
    const uint32_t swa = 2u * ((cl >> 3) & 3), swb = 2u * ((ol >> 3) & 3);
    const char *xplane = lds + cl * CSX * 16, *gplane = lds + Sh::XBYTES + ol * CSG * 16;
    f32x16 acc[9];
#pragma unroll
    for (int k = 0; k < 9; ++k)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[k][e] = 0.f;

    auto compute = [&](int bufno) {
        const char *xb = xplane + bufno * Sh::STAGE, *gb = gplane + bufno * Sh::STAGE;
#pragma unroll
        for (int i = 0; i < R; ++i) {
#pragma unroll
            for (int q = 0; q < NSEG; ++q) {
                const uint4 bvec = lds_read16(gb + (((uint32_t)(i * GV + 2 * q + m)) ^ swb) * 16);
#pragma unroll
                for (int r = 0; r < 3; ++r) {
                    const int row = i * S + r;
                    uint4 a0, a1, a2;
                    if (S == 1) {
                        const uint32_t v = (uint32_t)(row * CPV + 2 * q + m);
                        const uint4 v0 = lds_read16(xb + (v ^ swa) * 16), v1 = lds_read16(xb + ((v + 1) ^ swa) * 16);
                        a0 = v0;
                        a1 = window1(v0, v1);
                        a2 = window2(v0, v1);
                    } else {
                        const uint32_t e = (uint32_t)((row * 2) * CPV + 2 * q + m), o = e + CPV;
                        const uint4 v0 = lds_read16(xb + (e ^ swa) * 16), v1 = lds_read16(xb + ((e + 1) ^ swa) * 16);
                        a0 = v0;
                        a1 = lds_read16(xb + (o ^ swa) * 16);
                        a2 = window1(v0, v1);
                    }
                    acc[r * 3 + 0] = mfma32x32x16<DT>(a0, bvec, acc[r * 3 + 0]);
                    acc[r * 3 + 1] = mfma32x32x16<DT>(a1, bvec, acc[r * 3 + 1]);
                    acc[r * 3 + 2] = mfma32x32x16<DT>(a2, bvec, acc[r * 3 + 2]);
                }
            }
        }
    };

    // ---- zero both buffers once: the padding is never written again ------------------------------------------------
    for (int i = tid; i < 2 * Sh::STAGE / 16; i += 256) ((uint4 *)lds)[i] = make_uint4(0, 0, 0, 0);
    int b = sigma, h = 0;
    issue(b, h);
    __syncthreads();
    write(0);
    __syncthreads();
    for (int st = 0; st < nstages; ++st) {
        // the stage after this one (the last one once more at the end: written to the idle buffer, never read)
        if (st + 1 < nstages) {
            if (++h == H) { h = 0; b += p.nsplit; }
        }
        issue(b, h);
        compute(st & 1);
        write((st + 1) & 1);
        __syncthreads();
    }

    // ---- partial result: row (input channel) 8 (e / 4) + 4 (lane / 32) + e % 4, column (output channel) lane % 32 ----
    float *out = p.part + (size_t)sigma * 9 * p.CinP * p.CoutP;
    const int c0 = cb * 64 + (wave >> 1) * 32 + 4 * m, o = ob * 64 + (wave & 1) * 32 + (lane & 31);
#pragma unroll
    for (int k = 0; k < 9; ++k)
#pragma unroll
        for (int e = 0; e < 16; ++e)
            out[((size_t)k * p.CinP + c0 + 8 * (e >> 2) + (e & 3)) * p.CoutP + o] = acc[k][e];
}

template <int DT>
__device__ __forceinline__ float load_elem(const void *p, size_t i) {
    if (DT == SBNET_F32) return ((const float *)p)[i];
    const uint32_t bits = ((const uint16_t *)p)[i];
    return DT == SBNET_BF16 ? bf16_bits_to_float(bits) : unpack_lo<SBNET_F16>(bits);
}

// one thread per weight (tap, c, o); blockIdx.y is the split
template <int DT>
__global__ __launch_bounds__(256) void wgrad_direct(WgradParams p) {
    const int total = p.kh * p.kw * p.Cin * p.Cout;
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    int n = *p.count;
    if (n > p.cap) n = p.cap;
    const int sigma = blockIdx.y;
    if (sigma >= n) return;
    const int o = e % p.Cout, c = (e / p.Cout) % p.Cin, tap = e / (p.Cout * p.Cin);
    const int r = tap / p.kw, t = tap - r * p.kw;
    float acc = 0.f;
    for (int b = sigma; b < n; b += p.nsplit) {
        for (int i = 0; i < p.oh; ++i) {
            const size_t xrow = ((size_t)b * p.th + r + (size_t)p.sh * i) * p.tw + t;
            const size_t grow = ((size_t)b * p.oh + i) * p.ow;
            for (int j = 0; j < p.ow; ++j)
                acc = fmaf(load_elem<DT>(p.x, (xrow + (size_t)p.sw * j) * p.Cin + c), load_elem<DT>(p.g, (grow + j) * p.Cout + o), acc);
        }
    }
    p.part[(size_t)sigma * total + e] = acc;
}

// dw[tap][c][o] = partial results of the splits that had a tile, added in ascending order of the split
__global__ __launch_bounds__(256) void wgrad_sum(const float *__restrict__ part, const int32_t *__restrict__ count, int cap,
                                                 int nsplit, int taps, int Cin, int Cout, int CinP, int CoutP,
                                                 float *__restrict__ dw) {
    const int total = taps * Cin * Cout;
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    int n = *count;
    if (n > cap) n = cap;
    if (n > nsplit) n = nsplit;
    const int o = e % Cout, c = (e / Cout) % Cin, tap = e / (Cout * Cin);
    const size_t at = ((size_t)tap * CinP + c) * CoutP + o, step = (size_t)taps * CinP * CoutP;
    float acc = 0.f;
    int s = 0;
    for (; s + 4 <= n; s += 4) {
        const float a0 = part[at + (size_t)s * step], a1 = part[at + (size_t)(s + 1) * step];
        const float a2 = part[at + (size_t)(s + 2) * step], a3 = part[at + (size_t)(s + 3) * step];
        acc = ((acc + a0) + a1) + a2;
        acc += a3;
    }
    for (; s < n; ++s) acc += part[at + (size_t)s * step];
    dw[e] = acc;
}

struct WgradPlan {
    bool mfma;
    int s, nseg, nsplit, ncb, nob, CinP, CoutP;
    size_t part_bytes;
};

bool plan_wgrad(sbnet_dtype dt, int cap, int th, int tw, int Cin, int kh, int kw, int sh, int sw, int Cout, WgradPlan *q) {
    const int oh = (th - kh) / sh + 1, ow = (tw - kw) / sw + 1;
    const int taps = kh * kw;
    q->mfma = (dt == SBNET_BF16 || dt == SBNET_F16) && kh == 3 && kw == 3 && sh == sw && (sh == 1 || sh == 2) && Cin % 8 == 0 &&
              Cout % 8 == 0 && ow <= 32 && tw <= 32 * sw + 2 &&
              (long long)cap * th * tw * Cin * 2 < (1LL << 31) && (long long)cap * oh * ow * Cout * 2 < (1LL << 31);
    if (q->mfma) {
        q->s = sh;
        q->nseg = ow <= 16 && tw <= 16 * sw + 2 ? 1 : 2;
        q->ncb = (Cin + 63) / 64;
        q->nob = (Cout + 63) / 64;
        q->CinP = q->ncb * 64;
        q->CoutP = q->nob * 64;
        int ns = 256 / (q->ncb * q->nob);
        ns = ns / 8 * 8;                                   // splits of one channel block share an XCD's L2 with the others
        if (ns < 8) ns = 8;
        q->nsplit = ns;
    } else {
        q->s = q->nseg = 0;
        q->ncb = q->nob = 1;
        q->CinP = Cin;
        q->CoutP = Cout;
        const long long e = (long long)taps * Cin * Cout;
        if (e >= (1LL << 31)) return false;
        long long ns = (256LL * 1024 + e - 1) / e;
        if (ns > 1024) ns = 1024;
        q->nsplit = (int)ns;
    }
    if (q->nsplit > cap) q->nsplit = cap < 1 ? 1 : cap;
    q->part_bytes = (size_t)q->nsplit * taps * q->CinP * q->CoutP * sizeof(float);
    return true;
}

template <int DT, int S, int NSEG>
void launch_mfma(const WgradParams &p, hipStream_t s) {
    constexpr int bytes = 2 * WgradShape<S, NSEG>::STAGE;
    static_assert(bytes <= 160 * 1024, "two stages must fit in LDS");
    (void)hipFuncSetAttribute((const void *)wgrad_mfma<DT, S, NSEG>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    hipLaunchKernelGGL((wgrad_mfma<DT, S, NSEG>), dim3(p.nsplit * p.ncb * p.nob), dim3(256), bytes, s, p);
}

template <int DT>
void launch_mfma_dt(const WgradPlan &q, const WgradParams &p, hipStream_t s) {
    if (q.s == 1 && q.nseg == 1) launch_mfma<DT, 1, 1>(p, s);
    else if (q.s == 1) launch_mfma<DT, 1, 2>(p, s);
    else if (q.nseg == 1) launch_mfma<DT, 2, 1>(p, s);
    else launch_mfma<DT, 2, 2>(p, s);
}

}  // namespace

extern "C" size_t sbnet_conv_backward_weights_workspace_bytes(sbnet_dtype dtype, int cap, int th, int tw, int Cin, int kh,
                                                              int kw, int sh, int sw, int Cout) {
    if (!is_float_dtype(dtype) || cap < 0 || th < kh || tw < kw || kh <= 0 || kw <= 0 || sh <= 0 || sw <= 0 || Cin <= 0 ||
        Cout <= 0)
        return 0;
    WgradPlan q;
    if (!plan_wgrad(dtype, cap, th, tw, Cin, kh, kw, sh, sw, Cout, &q)) return 0;
    return (q.part_bytes + 255) / 256 * 256;
}

extern "C" sbnet_status sbnet_conv_on_tiles_backward_weights(const void *tiles_in, const void *dout_tiles, sbnet_dtype dtype,
                                                             const int32_t *count, int cap, int th, int tw, int Cin, int kh,
                                                             int kw, int sh, int sw, int Cout, float *dw, void *workspace,
                                                             size_t workspace_bytes, void *stream) {
    const char *who = "sbnet_conv_on_tiles_backward_weights";
    if (!tiles_in || !dout_tiles || !count || !dw || !workspace) return fail(SBNET_EINVAL, "%s: null pointer", who);
    if (!is_float_dtype(dtype)) return fail(SBNET_EUNSUPPORTED, "%s: dtype must be f32, bf16 or f16", who);
    if (cap < 0 || Cin <= 0 || Cout <= 0 || kh <= 0 || kw <= 0 || sh <= 0 || sw <= 0 || th < kh || tw < kw)
        return fail(SBNET_EINVAL, "%s: bad sizes", who);
    if (((uintptr_t)tiles_in | (uintptr_t)dout_tiles | (uintptr_t)workspace) & 15)
        return fail(SBNET_EINVAL, "%s: pointers must be 16-byte aligned", who);
    WgradPlan q;
    if (!plan_wgrad(dtype, cap, th, tw, Cin, kh, kw, sh, sw, Cout, &q)) return fail(SBNET_EUNSUPPORTED, "%s: too many weights", who);
    if (workspace_bytes < q.part_bytes) return fail(SBNET_EINVAL, "%s: workspace too small", who);
    hipStream_t s = (hipStream_t)stream;
    const int taps = kh * kw, total = taps * Cin * Cout;
    WgradParams p = {};
    p.x = tiles_in; p.g = dout_tiles; p.part = (float *)workspace; p.count = count;
    p.cap = cap; p.th = th; p.tw = tw; p.oh = (th - kh) / sh + 1; p.ow = (tw - kw) / sw + 1;
    p.Cin = Cin; p.Cout = Cout; p.kh = kh; p.kw = kw; p.sh = sh; p.sw = sw;
    p.nsplit = q.nsplit; p.ncb = q.ncb; p.nob = q.nob; p.CinP = q.CinP; p.CoutP = q.CoutP;
    p.x_tile_bytes = (uint32_t)((size_t)th * tw * Cin * 2);
    p.g_tile_bytes = (uint32_t)((size_t)p.oh * p.ow * Cout * 2);
    if (cap > 0) {
        if (q.mfma) {
            if (dtype == SBNET_BF16) launch_mfma_dt<SBNET_BF16>(q, p, s);
            else launch_mfma_dt<SBNET_F16>(q, p, s);
        } else {
            dim3 grid((unsigned)((total + 255) / 256), (unsigned)q.nsplit);
            if (dtype == SBNET_F32) hipLaunchKernelGGL(wgrad_direct<SBNET_F32>, grid, dim3(256), 0, s, p);
            else if (dtype == SBNET_BF16) hipLaunchKernelGGL(wgrad_direct<SBNET_BF16>, grid, dim3(256), 0, s, p);
            else hipLaunchKernelGGL(wgrad_direct<SBNET_F16>, grid, dim3(256), 0, s, p);
        }
        sbnet_status st = launch_status(who);
        if (st != SBNET_OK) return st;
    }
    hipLaunchKernelGGL(wgrad_sum, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const float *)workspace, count, cap,
                       q.nsplit, taps, Cin, Cout, q.CinP, q.CoutP, dw);
    return launch_status(who);
}

}  // namespace sbnet
