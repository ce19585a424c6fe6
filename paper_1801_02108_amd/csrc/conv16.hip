// 3x3, stride-1 tile convolution for output tiles whose sides are multiples of 16 pixels
// (Sec. 3.2 of arXiv 1801.02108: the regular convolution that runs on every gathered block;
// in fused mode also the gather before it and the scatter / scatter-add after it, Sec. 3.4).
//
// Design for gfx950, one workgroup (4 waves, one per SIMD) per CU, persistent over tiles:
//   * 32x32x16 MFMA: measured on MI355X, one wave per SIMD sustains ~88 % of the matrix peak with
//     this shape but only ~55 % with 16x16x32, and one wave per SIMD is what lets a wave own up
//     to 512 registers;
//   * weights stay in registers for the life of the workgroup: wave (rh, nh) owns output rows
//     rh*8..rh*8+7 of a 16x16 output sub-tile and output channels nh*32..nh*32+31 of the
//     workgroup's 64, i.e. 9*CIN/16 k-steps x 4 VGPRs (144 VGPRs at CIN = 64);
//   * the 18x18xCIN input sub-tile (block + halo) is double-buffered in LDS: the global loads of
//     the next tile are issued before the matrix work of the current one and written to the
//     other buffer after it, so HBM latency hides behind the MFMAs;
//   * an LDS fragment is 32 pixels (two consecutive input rows x 16 columns) x 16 channels; the
//     pixel stride is padded by 16 B, which makes the two rows of a fragment fall on disjoint
//     bank groups.  A fragment starting on an even row is used for tap rows 0 and 2 of two
//     neighbouring output row pairs, one starting on an odd row for tap row 1;
//   * consecutive work items map to the same XCD so that neighbouring tiles, which share halo
//     columns, hit in that XCD's L2.
#include "conv_common.h"

namespace sbnet {

constexpr int kT16 = 18;                 // input sub-tile side: 16 + 3 - 1
constexpr int kT16Px = kT16 * kT16;

struct Sub16 {
    int sub_h, sub_w;                    // 16x16 sub-tiles per block
    FastDiv div_sub, div_subw;
};

// one work item: a 16x16 output sub-tile of an active block
struct Item16 {
    uint32_t b;         // position in the index list
    int si, sj;         // sub-tile inside the block
    int n, by, bx;      // fused form: sample and block coordinates
};

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

template <int DT>
__device__ __forceinline__ f32x16 mfma32x32x16(uint4 a, uint4 b, f32x16 c) {
    if (DT == SBNET_BF16) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    } else {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
}

template <int DT, int CIN, bool FUSED>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void conv16_kernel(ConvParams p, Sub16 sp) {
    constexpr int KC = CIN / 16;                     // 16-channel k-steps per tap
    constexpr int CV = CIN / 8;                      // 16-byte vectors per pixel
    constexpr int PS = (CIN + 8) * 2;                // LDS bytes per pixel
    constexpr int NVEC = kT16Px * CV;
    constexpr int NV = (NVEC + 255) / 256;           // staging vectors per thread
    constexpr int KS = 9 * KC;
    constexpr int NST = 3 * KC;                      // pipeline stages: (tap column, channel step)
    __shared__ __align__(16) unsigned char lds[2][kT16Px * PS];

    const uint16_t *in = (const uint16_t *)p.in;
    uint16_t *out = (uint16_t *)p.out;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = lane >> 5, m = lane & 31;          // k-group / channel group, pixel within a fragment
    const int prow = m >> 4, pcol = m & 15;
    const int rh = wave >> 1, nh = wave & 1;
    const int ng = blockIdx.y;
    const uint32_t per_block = (uint32_t)sp.sub_h * sp.sub_w;
    const uint32_t G = gridDim.x;                    // multiple of 8
    // workgroups are dealt round-robin to the 8 XCDs: give each XCD a contiguous run of items
    const uint32_t first = (blockIdx.x & 7) * (G >> 3) + (blockIdx.x >> 3);

    auto decode = [&](uint32_t it) {
        Item16 c;
        c.b = fdiv(it, sp.div_sub);
        const uint32_t sidx = it - c.b * per_block;
        c.si = (int)fdiv(sidx, sp.div_subw);
        c.sj = (int)sidx - c.si * sp.sub_w;
        c.n = c.by = c.bx = 0;
        if (FUSED) {
            c.n = p.indices[3 * c.b];
            c.by = p.indices[3 * c.b + 1];
            c.bx = p.indices[3 * c.b + 2];
        }
        return c;
    };

    // The count and the first index triple are independent loads (the index is clamped into the
    // buffer), so their latencies overlap instead of chaining.
    const int nact_raw = *p.count;
    Item16 cur = decode(min(first, (uint32_t)p.cap * per_block - 1u));
    const uint32_t items = (uint32_t)min(nact_raw, p.cap) * per_block;
    if (first >= items) return;

    // ---- weights of this wave: every k-step of its 32 output channels
    uint4 wreg[KS];
    {
        const uint4 *wp = (const uint4 *)p.w + p.w32_offset + ((size_t)ng * KS * 2 + nh) * 64 + lane;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) wreg[ks] = wp[(size_t)ks * 128];
    }
    const int ch0 = ng * 64 + nh * 32 + g * 16;      // first of this lane's 16 output channels
    f32x16 biasv;
#pragma unroll
    for (int k = 0; k < 16; ++k) biasv[k] = 0.f;
    if (p.bias) {                                    // Cout % 8 == 0: eight at a time
#pragma unroll
        for (int h = 0; h < 2; ++h)
            if (ch0 + h * 8 < p.Cout) {
                const float4 b0 = *(const float4 *)(p.bias + ch0 + h * 8), b1 = *(const float4 *)(p.bias + ch0 + h * 8 + 4);
                biasv[h * 8 + 0] = b0.x; biasv[h * 8 + 1] = b0.y; biasv[h * 8 + 2] = b0.z; biasv[h * 8 + 3] = b0.w;
                biasv[h * 8 + 4] = b1.x; biasv[h * 8 + 5] = b1.y; biasv[h * 8 + 6] = b1.z; biasv[h * 8 + 7] = b1.w;
            }
    }
    // ReLU as an integer max on the float bits (negative floats are negative integers); without
    // ReLU the floor is INT_MIN and the max is the identity.  One VALU op, no NaN canonicalisation.
    const int floor_i = p.relu ? 0 : (int)0x80000000;

    // ---- per-thread staging plan, the same for every tile: element offset from the tile origin,
    //      (row, col) for the bounds test
    const int row_stride = (FUSED ? p.W : p.tw) * CIN;           // elements between tile rows in memory
    int goff[NV], rowcol[NV];
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        const int v = (int)threadIdx.x + k * 256;
        const int px = v / CV, c8 = v % CV;
        const int row = px / kT16, col = px % kT16;
        goff[k] = row * row_stride + col * CIN + c8 * 8;
        rowcol[k] = v < NVEC ? (row | (col << 8)) : 0xffff;      // row 255 never passes the test
    }

    uint4 stage[NV];
    auto fetch = [&](const Item16 &c) {
        // valid rows / columns of this sub-tile: inside the tile and (fused) inside the image
        int rlo = 0, rhi = min(kT16, p.th - c.si * 16), clo = 0, chi = min(kT16, p.tw - c.sj * 16);
        const uint16_t *base;
        if (FUSED) {
            const int gy0 = p.g_in.boffset_h + c.by * p.g_in.bstride_h + c.si * 16;
            const int gx0 = p.g_in.boffset_w + c.bx * p.g_in.bstride_w + c.sj * 16;
            rlo = max(0, -gy0); rhi = min(rhi, p.H - gy0);
            clo = max(0, -gx0); chi = min(chi, p.W - gx0);
            base = in + ((long long)c.n * p.H + gy0) * row_stride + (long long)gx0 * CIN;
        } else {
            base = in + ((long long)c.b * p.th + c.si * 16) * row_stride + (long long)c.sj * 16 * CIN;
        }
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const int row = rowcol[k] & 0xff, col = rowcol[k] >> 8;
            // A predicated load on purpose: written as an unconditional load from a selected address
            // (tile or a zero buffer) the compiler sinks every load down to its LDS store and a tile
            // costs NV memory round trips instead of one.
            stage[k] = make_uint4(0, 0, 0, 0);
            if (row >= rlo && row < rhi && col >= clo && col < chi) stage[k] = *(const uint4 *)(base + goff[k]);
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const int v = (int)threadIdx.x + k * 256;
            if (v < NVEC) *(uint4 *)(&lds[buf][(v / CV) * PS + (v % CV) * 16]) = stage[k];
        }
    };

    fetch(cur);
    stash(0);
    __syncthreads();

    int buf = 0;
    for (uint32_t it = first; it < items; it += G) {
        const uint32_t nit = it + G;
        const bool more = nit < items;
        Item16 nxt = cur;
        if (more) {
            nxt = decode(nit);
            fetch(nxt);
        }

        // ---- 16x16 outputs x 64 channels; this wave: 4 output row pairs x 32 channels.
        // Fragment j of a stage holds input rows rh*8 + j, rh*8 + j + 1 (j = 0..8) at tap column t;
        // output row pair P with tap row r reads fragment 2P + r.  Stages are software-pipelined:
        // while the matrix cores consume the nine fragments of one stage, the nine of the next are
        // read from LDS into the other register set; the scheduling barriers keep that interleaving.
        f32x16 acc[4];      // first MFMA of each accumulator starts from the bias
        const unsigned char *L = &lds[buf][((rh * 8 + prow) * kT16 + pcol) * PS + g * 16];
        uint4 xf[2][9];
#pragma unroll
        for (int j = 0; j < 9; ++j) xf[0][j] = *(const uint4 *)(L + (j * kT16) * PS);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int st = 0; st < NST; ++st) {
            const int t = st / KC, kc = st % KC;
            const int tn = (st + 1) / KC, kcn = (st + 1) % KC;
#pragma unroll
            for (int mm = 0; mm < 12; ++mm) {
                const int r = mm >> 2, P = mm & 3;             // P fastest: dependent MFMAs are 4 apart
                acc[P] = mfma32x32x16<DT>(wreg[(r * 3 + t) * KC + kc], xf[st & 1][2 * P + r],
                                          (st == 0 && r == 0) ? biasv : acc[P]);
                if (mm < 9 && st + 1 < NST)
                    xf[(st + 1) & 1][mm] = *(const uint4 *)(L + (mm * kT16 + tn) * PS + kcn * 32);
                __builtin_amdgcn_sched_barrier(0);
            }
        }

        // The next tile goes to the other LDS buffer before this tile's stores are issued: the
        // wait for its loads (issued a whole tile ago) is then not held up by store acknowledgements.
        if (more) stash(buf ^ 1);

        // ---- epilogue: ReLU, optional add, two 16-byte NHWC stores per pixel and lane
        {
            const int ocol = cur.sj * 16 + pcol;
            uint16_t *obase;
            long long orow_stride;
            bool col_ok = ocol < p.ow;
            int rlim = p.oh;                                   // rows [rmin, rlim) of the block are stored
            int rmin = 0;
            if (FUSED) {
                const int gy0 = p.g_out.boffset_h + cur.by * p.g_out.bstride_h;
                const int gx = p.g_out.boffset_w + cur.bx * p.g_out.bstride_w + ocol;
                col_ok = col_ok && gx >= 0 && gx < p.Wo;
                rlim = min(rlim, p.Ho - gy0);
                rmin = max(0, -gy0);
                orow_stride = (long long)p.Wo * p.Cout;
                obase = out + ((long long)cur.n * p.Ho + gy0) * orow_stride + (long long)gx * p.Cout + ch0;
            } else {
                orow_stride = (long long)p.ow * p.Cout;
                obase = out + (long long)cur.b * p.oh * orow_stride + (long long)ocol * p.Cout + ch0;
            }
#pragma unroll
            for (int P = 0; P < 4; ++P) {
                const int orow = cur.si * 16 + rh * 8 + 2 * P + prow;
                if (!(col_ok && orow >= rmin && orow < rlim)) continue;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    if (ch0 + h * 8 >= p.Cout) continue;       // Cout % 8 == 0: a vector is all in or all out
                    float v[8];
#pragma unroll
                    for (int k = 0; k < 8; ++k) v[k] = __int_as_float(max(__float_as_int(acc[P][h * 8 + k]), floor_i));
                    uint4 *d4 = (uint4 *)(obase + orow * orow_stride + h * 8);
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

        __syncthreads();
        buf ^= 1;
        cur = nxt;
    }
}

template <int DT, int CIN>
static void launch16(bool fused, const ConvParams &p, const Sub16 &sp, dim3 grid, hipStream_t s) {
    if (fused) hipLaunchKernelGGL((conv16_kernel<DT, CIN, true>), grid, dim3(256), 0, s, p, sp);
    else hipLaunchKernelGGL((conv16_kernel<DT, CIN, false>), grid, dim3(256), 0, s, p, sp);
}

bool conv16_try(sbnet_dtype dt, bool fused, const ConvParams &p, hipStream_t s, sbnet_status *st, const char *who) {
    if (dt != SBNET_BF16 && dt != SBNET_F16) return false;
    if (p.kh != 3 || p.kw != 3 || p.sh != 1 || p.sw != 1) return false;
    if (p.Cin != 32 && p.Cin != 64) return false;
    if (p.Cout % 8 != 0 || p.oh % 16 != 0 || p.ow % 16 != 0) return false;
    Sub16 sp;
    sp.sub_h = p.oh / 16;
    sp.sub_w = p.ow / 16;
    sp.div_sub = make_fastdiv((uint32_t)sp.sub_h * sp.sub_w);
    sp.div_subw = make_fastdiv((uint32_t)sp.sub_w);
    const long long items = (long long)p.cap * sp.sub_h * sp.sub_w;
    if (items >= (1LL << 31)) return false;
    // staging offsets inside one sub-tile are kept in 32-bit registers
    if (18LL * (fused ? p.W : p.tw) * p.Cin >= (1LL << 30)) return false;
    long long g = (items + 7) / 8 * 8;
    if (g > 256) g = 256;                             // one persistent workgroup per CU
    dim3 grid((unsigned)g, (unsigned)((p.Cout + 63) / 64));
    if (dt == SBNET_BF16) {
        if (p.Cin == 64) launch16<SBNET_BF16, 64>(fused, p, sp, grid, s);
        else launch16<SBNET_BF16, 32>(fused, p, sp, grid, s);
    } else {
        if (p.Cin == 64) launch16<SBNET_F16, 64>(fused, p, sp, grid, s);
        else launch16<SBNET_F16, 32>(fused, p, sp, grid, s);
    }
    *st = launch_status(who);
    return true;
}

}  // namespace sbnet
