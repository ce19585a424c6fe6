// Weight gradient of the tile convolution (training support for the convolution of Sec. 3.2 of arXiv 1801.02108):
//   dw[r][t][c][o] = sum over tiles b and output pixels (i, j) of x[b][r + sh i][t + sw j][c] * dout[b][i][j][o].
// The contraction runs over pixels, the one index that the channel-last tiles do not keep contiguous, and its result
// is small (kh kw Cin Cout numbers) while its inputs are the whole tile stacks.  So the tiles are split over many
// workgroups, each of which keeps a partial dw in registers for all its tiles and writes it once; a second kernel adds
// the partial results in a fixed order (no atomics: the result does not depend on scheduling).
//
// wgrad_mfma (3x3 or 1x1, stride 1 or 2, BF16/F16, channel counts multiples of 8): a workgroup owns 64 input by 64
// output channels, one 32x32 block per wave with one fp32 accumulator per tap (nine, or one).  Tiles pass through LDS a few output
// rows at a time (a "stage"), stored channel-major so that a lane's matrix operand (8 consecutive pixels of one
// channel) is one aligned 16-byte read:
//   * x rows are split by column phase (column % stride), so that the pixels a tap reads for consecutive output
//     pixels are consecutive; a tap's window starts 0 or 1 elements (stride 2) or 0, 1, 2 elements (stride 1) into a
//     16-byte vector and is cut from two neighbouring vectors with one byte-align per word;
//   * the channel planes are an odd number of 16-byte vectors apart and the vector index inside a plane is XOR-ed with
//     channel / 8: the 8-byte transposing writes of a wave (8 channel groups x 8 items of four pixels) and the
//     16-byte operand reads (consecutive channels) both spread over all banks; the spare vector at the end of each
//     plane takes the writes of staging slots that hold nothing, so that the writes need no branch;
//   * columns beyond the output row and rows beyond the tile hold zeros, in both operands, so that a partial row or
//     stage adds nothing.
// Stages alternate between two LDS buffers: the loads of the next stage are issued at the top of a stage, and in its
// second half their data, transposed in registers four pixels at a time, is written to the other buffer between the
// matrix instructions.
//
// wgrad_direct: every other shape and fp32; one thread per weight, plain loops.
#include <hip/hip_runtime.h>

#include "conv_common.h"

namespace sbnet {
namespace {

struct WgradParams {
    const void *x;            // [cap][th][tw][Cin]
    const void *g;            // [cap][oh][ow][Cout]
    float *part;              // [nsplit][taps][CinP][CoutP], split_stride() floats from one split to the next
    const int32_t *count;
    int cap, th, tw, oh, ow, Cin, Cout, kh, kw, sh, sw;
    int nsplit, ncb, nob, CinP, CoutP;
    int split_factor;         // splits used = min(nsplit, n, split_factor * sqrt(n))
    uint32_t x_tile_bytes, g_tile_bytes;
};

template <int KH, int S, int NSEG>
struct WgradShape {
    static constexpr int R = 8 / (S * NSEG);              // output rows per stage
    static constexpr int RX = (R - 1) * S + KH;           // input rows per stage
    // 16-byte vectors per phase row of x: 3x3 keeps one spare for the window of the taps; 1x1 reads 16 NSEG pixels only
    static constexpr int CPV = KH == 1 ? 2 * NSEG : 2 * NSEG + 1;
    static constexpr int XPL = (RX * S * CPV + 7) / 8 * 8;
    static constexpr int CSX = XPL + 1;                   // vectors between channel planes of x (odd)
    static constexpr int GV = 2 * NSEG;                   // vectors per row of dout
    static constexpr int GPL = (R * GV + 7) / 8 * 8;
    static constexpr int CSG = GPL + 1;
    static constexpr int XBYTES = 64 * CSX * 16;
    static constexpr int STAGE = 64 * (CSX + CSG) * 16;
    // staging items: four pixels of one phase row (or of one row of dout) times 8 channels
    static constexpr int QX = KH == 1 ? 4 * NSEG : (16 * NSEG + 2 + 3) / 4;    // items per phase row of x (at most 16 NSEG + KH - 1 pixels)
    static constexpr int QG = 4 * NSEG;                   // items per row of dout
    static constexpr int NIX = (RX * S * QX * 8 + 255) / 256;
    static constexpr int NIG = (R * QG * 8 + 255) / 256;
};

// Floats between the partial results of consecutive splits: the size of one result plus 256 bytes.  All workgroups
// write their results at the same time and at the same offsets inside them; with the bare size (a multiple of 16 KiB
// for 64 x 64 blocks) between them those writes would all fall on a few memory channels.
__host__ __device__ __forceinline__ size_t split_stride(int taps, int CinP, int CoutP) { return (size_t)taps * CinP * CoutP + 64; }

// Splits actually used for n active tiles, of the nsplit the launch provides.  Every split costs a partial result
// (written once, read once by the sum) and every tile of a split costs matrix time, so the best number grows with the
// square root of n: 8 sqrt(n) suits the two costs measured on 64 x 64 channel blocks.  Both kernels call this with
// the same arguments.
__device__ __forceinline__ int splits_used(int n, int nsplit, int factor) {
    int ns = (int)sqrtf((float)(factor * factor) * (float)n);     // factor: 8 for 3x3; a 1x1 partial result is a ninth of that: 16
    if (ns > n) ns = n;
    if (ns > nsplit) ns = nsplit;
    return ns < 1 ? 1 : ns;
}

__device__ __forceinline__ uint4 lds_read16(const char *p) { return *(const uint4 *)p; }

// elements 1..8 of the 16 elements in (v0, v1)
__device__ __forceinline__ uint4 window1(uint4 v0, uint4 v1) {
    return make_uint4(__builtin_amdgcn_alignbyte(v0.y, v0.x, 2), __builtin_amdgcn_alignbyte(v0.z, v0.y, 2),
                      __builtin_amdgcn_alignbyte(v0.w, v0.z, 2), __builtin_amdgcn_alignbyte(v1.x, v0.w, 2));
}
// elements 2..9
__device__ __forceinline__ uint4 window2(uint4 v0, uint4 v1) { return make_uint4(v0.y, v0.z, v0.w, v1.x); }

// two 16-bit halves, one from each word: (lo, lo) or (hi, hi)
__device__ __forceinline__ uint32_t pair_lo(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ uint32_t pair_hi(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

template <int DT, int KH, int S, int NSEG>
__global__ __launch_bounds__(256) void wgrad_mfma(WgradParams p) {
    typedef WgradShape<KH, S, NSEG> Sh;
    constexpr int TAPS = KH * KH;
    constexpr int R = Sh::R, RX = Sh::RX, CPV = Sh::CPV, CSX = Sh::CSX, CSG = Sh::CSG, GV = Sh::GV;
    constexpr int NIX = Sh::NIX, NIG = Sh::NIG, NI = NIX + NIG, QX = Sh::QX, QG = Sh::QG;
    extern __shared__ __align__(16) char lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sigma = blockIdx.x % p.nsplit, cbob = blockIdx.x / p.nsplit;
    const int cb = cbob / p.nob, ob = cbob - cb * p.nob;
    int n = *p.count;
    if (n > p.cap) n = p.cap;
    const int ns = splits_used(n, p.nsplit, p.split_factor);
    if (n <= 0 || sigma >= ns) return;                             // the sum reads no partial result of this split
    const int ntiles = (n - sigma + ns - 1) / ns;
    const int H = (p.oh + R - 1) / R;
    const int nstages = ntiles * H;

    // ---- what this thread stages, fixed for the whole kernel: items of four pixels (consecutive in a phase row of x,
    // or in a row of dout) by 8 channels = four 16-byte loads, transposed in registers into 8 writes of four pixels.
    // rel: byte offset of the first pixel inside the stage's first row (kOutOfRange: no item); cnt: pixels that exist.
    uint32_t rel[NI], at[NI], cnt[NI];
    const int cv = tid & 7;                                        // 8-channel group inside the workgroup's 64
#pragma unroll
    for (int u = 0; u < NIX; ++u) {
        const int it = (u * 256 + tid) >> 3;
        const int q = it % QX, rp = it / QX, ph = rp % S, ry = rp / S;
        const int x = 4 * q * S + ph;                              // column of the item's first pixel
        const bool ok = ry < RX && cb * 64 + cv * 8 < p.Cin && x < p.tw;
        rel[u] = ok ? (uint32_t)(((ry * p.tw + x) * p.Cin + cb * 64 + cv * 8) * 2) : kOutOfRange;
        cnt[u] = ok ? (uint32_t)((p.tw - x + S - 1) / S) : 0u;
        const uint32_t v = (uint32_t)((ry * S + ph) * CPV + (q >> 1)) ^ (uint32_t)cv;
        at[u] = (uint32_t)(cv * 8 * CSX * 16) + (ok ? v * 16 + (q & 1) * 8 : (uint32_t)Sh::XPL * 16);
    }
#pragma unroll
    for (int u = 0; u < NIG; ++u) {
        const int it = (u * 256 + tid) >> 3;
        const int q = it % QG, gy = it / QG, x = 4 * q;
        const bool ok = gy < R && ob * 64 + cv * 8 < p.Cout && x < p.ow;
        rel[NIX + u] = ok ? (uint32_t)(((gy * p.ow + x) * p.Cout + ob * 64 + cv * 8) * 2) : kOutOfRange;
        cnt[NIX + u] = ok ? (uint32_t)(p.ow - x) : 0u;
        const uint32_t v = (uint32_t)(gy * GV + (q >> 1)) ^ (uint32_t)cv;
        at[NIX + u] = (uint32_t)(Sh::XBYTES + cv * 8 * CSG * 16) + (ok ? v * 16 + (q & 1) * 8 : (uint32_t)Sh::GPL * 16);
    }
    const uint32_t x_stage_step = (uint32_t)(R * S * p.tw * p.Cin * 2), g_stage_step = (uint32_t)(R * p.ow * p.Cout * 2);
    const uint32_t x_px_step = (uint32_t)(S * p.Cin * 2), g_px_step = (uint32_t)(p.Cout * 2);

    uint4 staged[NI][4];
    auto issue = [&](int b, int h) {
        // one buffer descriptor per tile: offsets stay below the tile size whatever the size of the stack, and an
        // offset beyond the tile (a row past its last one) reads zeros by itself
        const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(
            (void *)((const char *)p.x + (size_t)b * p.x_tile_bytes), 0, (int)p.x_tile_bytes, kBufWord3);
        const __amdgpu_buffer_rsrc_t gr = __builtin_amdgcn_make_buffer_rsrc(
            (void *)((const char *)p.g + (size_t)b * p.g_tile_bytes), 0, (int)p.g_tile_bytes, kBufWord3);
#pragma unroll
        for (int u = 0; u < NI; ++u) {
            const bool isx = u < NIX;
            const uint32_t o = (uint32_t)h * (isx ? x_stage_step : g_stage_step) + rel[u];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // pixels beyond the row's end (a slot that holds nothing has cnt = 0): zeros; so are, by the
                // descriptor, pixels beyond the tile (rows past its last one, the rest of a last row it does not fill)
                const uint32_t oj = o + j * (isx ? x_px_step : g_px_step);
                const uint32_t off = (uint32_t)j < cnt[u] ? oj : kOutOfRange;
                staged[u][j] = buf_load16(isx ? xr : gr, off);
            }
        }
    };
    // channel k of item u: its four pixels as one 8-byte write into channel plane k of the item's 8
    auto write_elem = [&](int w, char *base) {
        const int u = w >> 3, k = w & 7;
        uint32_t word[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint4 d = staged[u][j];
            word[j] = (k >> 1) == 0 ? d.x : (k >> 1) == 1 ? d.y : (k >> 1) == 2 ? d.z : d.w;
        }
        uint2 v;
        v.x = (k & 1) ? pair_hi(word[0], word[1]) : pair_lo(word[0], word[1]);
        v.y = (k & 1) ? pair_hi(word[2], word[3]) : pair_lo(word[2], word[3]);
        *(uint2 *)(base + at[u] + k * ((u < NIX ? CSX : CSG) * 16)) = v;
    };

    // ---- matrix operands of this wave ------------------------------------------------------------------------------
    const int cl = (wave >> 1) * 32 + (lane & 31), ol = (wave & 1) * 32 + (lane & 31), m = lane >> 5;
    const uint32_t swa = (uint32_t)(cl >> 3), swb = (uint32_t)(ol >> 3);
    const char *xplane = lds + cl * CSX * 16, *gplane = lds + Sh::XBYTES + ol * CSG * 16;
    f32x16 acc[TAPS];
#pragma unroll
    for (int k = 0; k < TAPS; ++k)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[k][e] = 0.f;

    // one step = 16 output pixels of one row (segment q of row i; q is the outer index so that consecutive steps share
    // input rows): the operand of dout and, per kernel row, the vectors the three taps are cut from.  A step reads
    // only the input rows the step before did not have.
    constexpr int T = R * NSEG, XV = S == 1 ? 2 : 3;
    struct Ops { uint4 b, x[KH][XV]; };
    auto load_row = [&](Ops &o, const char *xb, int i, int q, int r) {
        const uint32_t v = (uint32_t)((i * S + r) * S * CPV + 2 * q + m);          // phase 0 of the row
        o.x[r][0] = lds_read16(xb + (v ^ swa) * 16);
        if (KH == 1) return;                                                       // the one tap is vector 0
        o.x[r][1] = lds_read16(xb + ((v + 1) ^ swa) * 16);
        if (S == 2) o.x[r][XV - 1] = lds_read16(xb + ((v + CPV) ^ swa) * 16);      // phase 1
    };
    auto load_ops = [&](Ops &o, const Ops &prev, int bufno, int t) {
        const char *xb = xplane + bufno * Sh::STAGE, *gb = gplane + bufno * Sh::STAGE;
        const int q = t / R, i = t - q * R;
        o.b = lds_read16(gb + (((uint32_t)(i * GV + 2 * q + m)) ^ swb) * 16);
#pragma unroll
        for (int r = 0; r < KH; ++r) {
            if (i > 0 && r + S < KH) {
#pragma unroll
                for (int k = 0; k < XV; ++k) o.x[r][k] = prev.x[r + S][k];
            } else {
                load_row(o, xb, i, q, r);
            }
        }
    };
    auto mfma1 = [&](const Ops &o, int j) {                       // tap j = 3 r + t of this step
        const int r = j / KH, t = j - KH * r;
        uint4 a;
        if (S == 1) a = t == 0 ? o.x[r][0] : t == 1 ? window1(o.x[r][0], o.x[r][1]) : window2(o.x[r][0], o.x[r][1]);
        else a = t == 0 ? o.x[r][0] : t == 1 ? o.x[r][XV - 1] : window1(o.x[r][0], o.x[r][1]);
        acc[j] = mfma32x32x16<DT>(a, o.b, acc[j]);
    };

    // stages in order: (tile sigma, rows 0..R-1), (tile sigma, rows R..), ..., (tile sigma + ns, rows 0..), ...
    int b = sigma, h = 0, issued = 0;
    auto next_stage = [&]() {                                      // beyond the last stage: the last one again
        if (issued + 1 < nstages) {
            ++issued;
            if (++h == H) { h = 0; b += ns; }
        }
    };

    // ---- zero both buffers once: the padding is never written again ------------------------------------------------
    issue(b, h);
    for (int i = tid; i < 2 * Sh::STAGE / 16; i += 256) ((uint4 *)lds)[i] = make_uint4(0, 0, 0, 0);
    __syncthreads();
#pragma unroll
    for (int w = 0; w < NI * 8; ++w) write_elem(w, lds);
    __syncthreads();
    for (int st = 0; st < nstages; ++st) {
        // loads of the next stage at the top; matrix work on buffer st % 2, the operands of a step read one step ahead;
        // in the second half of the stage the loaded items go to the other buffer, between the matrix instructions
        next_stage();
        issue(b, h);
        const int cur = st & 1;
        char *other = lds + (cur ^ 1) * Sh::STAGE;
        Ops o0, o1;
        load_ops(o0, o0, cur, 0);
#pragma unroll
        for (int t = 0; t < T; ++t) {
            Ops &now = (t & 1) ? o1 : o0, &nxt = (t & 1) ? o0 : o1;
            if (t + 1 < T) load_ops(nxt, now, cur, t + 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < TAPS; ++j) {
                mfma1(now, j);
                constexpr int W = NI * 8, SLOTS = T * TAPS, FIRST = SLOTS / 2, LATE = SLOTS - FIRST;
                const int slot = t * TAPS + j - FIRST;
                if (slot >= 0) {
#pragma unroll
                    for (int w = (slot * W + LATE - 1) / LATE; w < ((slot + 1) * W + LATE - 1) / LATE; ++w) write_elem(w, other);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __syncthreads();
    }

    // ---- partial result.  A lane holds column (output channel) lane % 32 and rows (input channels)
    // 8 (e / 4) + 4 (lane / 32) + e % 4 of its wave's 32 x 32 block; written like that, every store instruction would
    // carry 4 bytes per lane.  Each block goes through a wave-private LDS tile (the stage buffers are free now: the loop
    // ends with a barrier) and leaves as 16-byte stores along the output channels.
    float *out = p.part + (size_t)sigma * split_stride(TAPS, p.CinP, p.CoutP);
    constexpr int TS = 36;                                         // floats per tile row: 16-byte aligned rows, shifted banks
    float *tiles = (float *)lds + wave * (2 * 32 * TS);
    const int cblk = cb * 64 + (wave >> 1) * 32, oblk = ob * 64 + (wave & 1) * 32;
#pragma unroll
    for (int k = 0; k < TAPS; ++k) {
        float *t = tiles + (k & 1) * (32 * TS);
#pragma unroll
        for (int e = 0; e < 16; ++e) t[(8 * (e >> 2) + 4 * m + (e & 3)) * TS + (lane & 31)] = acc[k][e];
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
            const int row = pass * 8 + (lane >> 3), col = 4 * (lane & 7);
            const float4 v = *(const float4 *)(t + row * TS + col);
            *(float4 *)(out + ((size_t)k * p.CinP + cblk + row) * p.CoutP + oblk + col) = v;
        }
        __builtin_amdgcn_wave_barrier();
    }
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
    const int sigma = blockIdx.y, ns = splits_used(n, p.nsplit, p.split_factor);
    if (n <= 0 || sigma >= ns) return;
    const int o = e % p.Cout, c = (e / p.Cout) % p.Cin, tap = e / (p.Cout * p.Cin);
    const int r = tap / p.kw, t = tap - r * p.kw;
    float acc = 0.f;
    for (int b = sigma; b < n; b += ns) {
        for (int i = 0; i < p.oh; ++i) {
            const size_t xrow = ((size_t)b * p.th + r + (size_t)p.sh * i) * p.tw + t;
            const size_t grow = ((size_t)b * p.oh + i) * p.ow;
            for (int j = 0; j < p.ow; ++j)
                acc = fmaf(load_elem<DT>(p.x, (xrow + (size_t)p.sw * j) * p.Cin + c), load_elem<DT>(p.g, (grow + j) * p.Cout + o), acc);
        }
    }
    p.part[(size_t)sigma * split_stride(p.kh * p.kw, p.CinP, p.CoutP) + e] = acc;
}

// dw[tap][c][o] = partial results of the splits that had a tile, added in a fixed order: the NW waves of a workgroup
// each add every NW-th split in ascending order (many independent loads in flight, where one chain of dependent
// loads would be bound by latency), then the NW sums are added in ascending order of the wave.  NW = 16 where the
// weights fill at most 256 workgroups (1x1 kernels: the launch is short and the splits are many), else 4.
template <int NW>
__global__ __launch_bounds__(64 * NW) void wgrad_sum(const float *__restrict__ part, const int32_t *__restrict__ count, int cap,
                                                  int nsplit, int split_factor, int taps, int Cin, int Cout, int CinP,
                                                  int CoutP, float *__restrict__ dw) {
    __shared__ float slice[NW][64];
    const int total = taps * Cin * Cout;
    const int lane = threadIdx.x & 63, k = threadIdx.x >> 6;
    const int e = blockIdx.x * 64 + lane;
    int n = *count;
    if (n > cap) n = cap;
    n = n > 0 ? splits_used(n, nsplit, split_factor) : 0;
    float acc = 0.f;
    if (e < total) {
        const int o = e % Cout, c = (e / Cout) % Cin, tap = e / (Cout * Cin);
        const size_t at = ((size_t)tap * CinP + c) * CoutP + o, step = split_stride(taps, CinP, CoutP);
        // batches of 8 loads in flight (splits beyond the last read as the first one and count as zero)
        for (int s = k; s < n; s += 8 * NW) {
            float a[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int sj = s + NW * j;
                const float v = part[at + (size_t)(sj < n ? sj : 0) * step];
                a[j] = sj < n ? v : 0.f;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) acc += a[j];
        }
    }
    slice[k][lane] = acc;
    __syncthreads();
    if (k == 0 && e < total) {
        float t = slice[0][lane];
#pragma unroll
        for (int i = 1; i < NW; ++i) t += slice[i][lane];
        dw[e] = t;
    }
}

struct WgradPlan {
    bool mfma;
    int kh, s, nseg, nsplit, ncb, nob, CinP, CoutP;
    bool flat;               // 1x1 at stride 1: the tile as one run of pixels
    size_t part_bytes;
};

bool plan_wgrad(sbnet_dtype dt, int cap, int th, int tw, int Cin, int kh, int kw, int sh, int sw, int Cout, WgradPlan *q) {
    const int oh = (th - kh) / sh + 1, ow = (tw - kw) / sw + 1;
    const int taps = kh * kw;
    q->flat = kh == 1 && kw == 1 && sh == 1 && sw == 1;
    q->mfma = (dt == SBNET_BF16 || dt == SBNET_F16) && (kh == 3 || kh == 1) && kw == kh && sh == sw && (sh == 1 || sh == 2) && Cin % 8 == 0 &&
              Cout % 8 == 0 && (q->flat || (ow <= 32 && tw <= 32 * sw + 2)) &&
              (long long)th * tw * Cin * 2 < (1LL << 30) && (long long)oh * ow * Cout * 2 < (1LL << 30);
    q->kh = kh;
    if (q->mfma) {
        q->s = sh;
        q->nseg = q->flat || (ow <= 16 && tw <= 16 * sw + 2) ? 1 : 2;
        q->ncb = (Cin + 63) / 64;
        q->nob = (Cout + 63) / 64;
        q->CinP = q->ncb * 64;
        q->CoutP = q->nob * 64;
        // one workgroup per CU for 3x3 (its two stages take 100 KB of LDS); two for 1x1 (70 KB), whose stages hold
        // little matrix work and wait on memory: the second workgroup's loads fill that wait
        int ns = (kh == 1 ? 512 : 256) / (q->ncb * q->nob);
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
    q->part_bytes = (size_t)q->nsplit * split_stride(taps, q->CinP, q->CoutP) * sizeof(float);
    return true;
}

template <int DT, int KH, int S, int NSEG>
void launch_mfma(const WgradParams &p, hipStream_t s) {
    constexpr int bytes = 2 * WgradShape<KH, S, NSEG>::STAGE;
    static_assert(bytes <= 160 * 1024, "two stages must fit in LDS");
    (void)hipFuncSetAttribute((const void *)wgrad_mfma<DT, KH, S, NSEG>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    hipLaunchKernelGGL((wgrad_mfma<DT, KH, S, NSEG>), dim3(p.nsplit * p.ncb * p.nob), dim3(256), bytes, s, p);
}

template <int DT>
void launch_mfma_dt(const WgradPlan &q, const WgradParams &p, hipStream_t s) {
    if (q.kh == 3) {
        if (q.s == 1 && q.nseg == 1) launch_mfma<DT, 3, 1, 1>(p, s);
        else if (q.s == 1) launch_mfma<DT, 3, 1, 2>(p, s);
        else if (q.nseg == 1) launch_mfma<DT, 3, 2, 1>(p, s);
        else launch_mfma<DT, 3, 2, 2>(p, s);
    } else {
        if (q.s == 1 && q.nseg == 1) launch_mfma<DT, 1, 1, 1>(p, s);
        else if (q.s == 1) launch_mfma<DT, 1, 1, 2>(p, s);
        else if (q.nseg == 1) launch_mfma<DT, 1, 2, 1>(p, s);
        else launch_mfma<DT, 1, 2, 2>(p, s);
    }
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
    const sbnet_tuning tune = tuning();
    p.split_factor = taps == 1 ? tune.wgrad_split_factor_1x1 : tune.wgrad_split_factor_3x3;
    p.x_tile_bytes = (uint32_t)((size_t)th * tw * Cin * 2);
    p.g_tile_bytes = (uint32_t)((size_t)p.oh * p.ow * Cout * 2);
    if (q.mfma && q.flat) {
        // 1x1 at stride 1 pairs pixel with pixel, whatever the tile's shape: the matrix kernel sees rows of 16 pixels
        // (the tile sizes in bytes stay the true ones, so the pixels past the end of the last row read as zeros)
        p.th = p.oh = (th * tw + 15) / 16;
        p.tw = p.ow = 16;
    }
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
    const unsigned sum_grid = (unsigned)((total + 63) / 64);
    if (sum_grid <= 256)
        hipLaunchKernelGGL(wgrad_sum<16>, dim3(sum_grid), dim3(1024), 0, s, (const float *)workspace, count, cap, q.nsplit, p.split_factor,
                           taps, Cin, Cout, q.CinP, q.CoutP, dw);
    else
        hipLaunchKernelGGL(wgrad_sum<4>, dim3(sum_grid), dim3(256), 0, s, (const float *)workspace, count, cap, q.nsplit, p.split_factor,
                           taps, Cin, Cout, q.CinP, q.CoutP, dw);
    return launch_status(who);
}

}  // namespace sbnet
