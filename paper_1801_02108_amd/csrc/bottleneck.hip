// Sparse residual (bottleneck) unit on tiles (Sec. 3.3, Fig. 4 of arXiv 1801.02108): the three
// convolutions of a ResNet bottleneck (1x1 C->Cm + ReLU, 3x3 Cm->Cm + ReLU, 1x1 Cm->C; batch norm
// folded into weights and bias) share one gather and one scatter-add (Sec. 3.4).  C is 64, 96, 128, 192 or
// 256 with Cm any multiple of 8 up to 64 (a narrower unit runs as width 64 on zero-padded weights), or 384
// with Cm in 72 .. 96: the widths of the four stages of the detector backbone of Sec. 4.  The receptive
// field of the whole unit is that of its single 3x3, so the input tile is block + 1-pixel halo.  The same
// kernel, with a stride of 2 in the 3x3, more output than input channels and a projected shortcut, is the
// downsampling unit that opens a stage (template parameters S, PROJ, CO below).
//
// One kernel per unit; per TS x TS output sub-tile (TS = 16, or 8 for blocks that are no multiple of 16
// and for problems with too few 16x16 sub-tiles to occupy the device) and workgroup (4 waves, one per
// SIMD).  W1 and the biases stay in LDS for the life of the workgroup (MFMA operand order).  16-pixel
// sub-tiles keep W3 there too and re-read W2 (the 3x3, 72 KB) from L2 for every tile, through a ring of
// registers a few stages ahead of P2's matrix work; 8-pixel sub-tiles keep W2 in LDS and read W3 from L2:
//   P1  t1 = ReLU(W1 x + b1) on the (TS+2)^2 input sub-tile.  x passes through LDS in 64-channel
//       chunks: eight lanes read one pixel's 128 contiguous bytes (8 full cache lines per wave
//       instruction; loading the 32x32x16 B operand directly touches 32 lines for the same 1 KB and
//       runs at the L1 tag rate), two chunks are in flight in registers;
//       t1 goes to LDS as bf16/f16.  Positions outside the image are forced to zero: the dense
//       network pads the 3x3's input, i.e. t1, with zeros, and ReLU(b1) is not zero.  While the chunk
//       that holds a wave's output channels lies in LDS, the wave copies the block's own pixels of it to
//       registers as MFMA B operands: the residual never leaves the chip (the pre-activation form,
//       whose LDS copy is the transformed x, requests x again in the middle of P1, while the same
//       cache lines are passing through L2).  The next tile's first chunk is requested a few vectors
//       at a time while t1 is written, its second one vector per stage of P2.
//   P2  t2 = ReLU(W2 * t1 + b2), the 3x3 as nine shifted reads of the LDS copy of t1 (same scheme
//       as the stand-alone 3x3 tile kernel); t2 goes to LDS.
//   P3  t3 = W3 t2 + b3; fused form: y = x + t3 on the block's pixels; on-tiles form: t3 is stored.
//       A wave owns 64 (or 32) neighbouring output channels.  The bias enters by a matrix step (three
//       bf16 / f16 pieces of each fp32 bias against a column of ones) and the residual by two more
//       against a 0/1 matrix, so the sum is formed in fp32 and rounded once, and the phase, which is
//       bound by its LDS traffic, reads neither from LDS.  In the MFMA result layout a lane holds
//       16 channels of one pixel, so stores from it would be 16-byte pieces 2*C bytes apart, one
//       memory request each.  The results are therefore rounded to the storage type and transposed
//       through a wave-private LDS area (the space of t1, dead by then): eight neighbouring lanes
//       then hold the wave's 128 contiguous bytes of one pixel and store whole cache lines per
//       request, non-temporal.  (The pre-activation form adds its residual in that layout.)
// Global memory is reached through buffer descriptors that cover one sample (or one tile): rows outside
// the image fall outside the descriptor, columns outside get an out-of-range offset, and the hardware
// returns zeros for such loads and drops such stores, so no memory operation needs a branch or predicate.
// HBM traffic per sub-tile is the input tile once and the output block once.
#include <type_traits>

#include "conv_common.h"

namespace sbnet {

constexpr int kCm = 64;                  // bottleneck width
constexpr int kPS = (kCm + 8) * 2;       // LDS bytes per pixel of t1 / t2 (16 B pad)

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16b;

template <int DT>
__device__ __forceinline__ f32x16b mfma32(uint4 a, uint4 b, f32x16b c) {
    if (DT == SBNET_BF16) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    } else {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
}

struct BneckParams {
    const void *in;              // fused: x [N][H][W][C]; on-tiles: tiles [cap][th][tw][C]
    void *out;                   // fused: y [N][H][W][C]; on-tiles: t3 tiles [cap][bo_h][bo_w][C]
    const void *w1, *w2, *w3;    // packed weights (32x32x16 operand copies are used)
    size_t w1_off, w2_off, w3_off;   // start of those copies, in 16-byte units
    const float *b1, *b2, *b3;
    const int32_t *indices, *count;
    int cap;
    int th, tw, oh, ow;          // tile and output block extents
    int H, W;                    // input image extent (border zeroing; fused addressing)
    int Ho, Wo;                  // output image extent (fused addressing; equal to H, W without a stride)
    const void *ws;              // downsampling form: packed 1x1 shortcut weights C -> CO (32x32x16 operand copy at ws_off)
    size_t ws_off;
    const float *bs;             // ... and its bias
    sbnet_geom g_in, g_out;
    int sub_h, sub_w;
    FastDiv div_sub, div_subw;
    // Which sub-tile size runs is decided on the device, from the count of active blocks: rounds of work over the
    // workgroups with either size, an 8 x 8 item costing cost8 eighths of a 16 x 16 one.  The host cannot see the
    // count, so it launches both variants and the one the rule does not pick returns at once (want16 says which
    // variant this launch is; per16 / per8 = sub-tiles per block of either size, per16 = 0: 8 x 8 only).
    int per16, per8, cost8, want16;
    const float *pre_scale, *pre_shift;   // pre-activation ReLU(scale * x + shift) in front of conv1, or both null
    // Bottleneck widths below 64 run as width 64: the packed weights carry zeros for the channels that do not
    // exist (t1 and t2 are exactly zero there), the biases are read as zero beyond Cm, and the packed copies of
    // W2 and W3 hold km = (Cm rounded up to 32) / 16 k-steps per tap instead of 4.
    int Cm, km;
};

struct BItem {
    uint32_t b;
    int si, sj, n, by, bx;
};

constexpr uint32_t kBufWord3B = 0x00020000u;     // raw buffer descriptor, 32-bit data format
constexpr uint32_t kOutOfRangeB = 0x80000000u;   // offset beyond any descriptor this kernel builds
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4b;
typedef const u32x4b __attribute__((address_space(1))) *gvec_t;    // a pointer known to be to global memory
__device__ __forceinline__ uint4 gload16(gvec_t q) {
    const u32x4b v = *q;
    return make_uint4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ uint4 bload16(__amdgpu_buffer_rsrc_t r, uint32_t off) {
    const u32x4b v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0);
    return make_uint4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void bstore16(__amdgpu_buffer_rsrc_t r, uint32_t off, uint4 d) {
    u32x4b v;
    v[0] = d.x; v[1] = d.y; v[2] = d.z; v[3] = d.w;
    // non-temporal: the results are not read again by this kernel and should not push the input, whose block
    // pixels are read a second time as the residual, out of L2
    __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)off, 0, 2);
}

__device__ __forceinline__ int relu_bits(float v) { return max(__float_as_int(v), 0); }

// ReLU of two values and their rounding to the storage type, in that word's two halves.  Rounding keeps the sign, so
// the ReLU is taken afterwards, on both halves at once: a negative bf16 / f16 (or -0) is a negative 16-bit integer.
typedef short short2b __attribute__((ext_vector_type(2)));
template <int DT>
__device__ __forceinline__ uint32_t relu_pack2(float lo, float hi) {
    const short2b v = __builtin_bit_cast(short2b, pack2<DT>(lo, hi)), zero = {0, 0};
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(v, zero));
}

// S, PROJ, CO: the downsampling form (Sec. 4: the units that open a stage): the 3x3 runs with stride S = 2 on the
// (2 TS + 1)^2 input sub-tile of Fig. 3, the unit has CO output channels and its shortcut is the 1x1 convolution
// with the same stride (PROJ), whose products P3 adds to the same accumulators as W3 t2: K is simply longer by C.
// Its B operands are the input pixels under the output pixels, read from L2 in the MFMA layout (they passed
// through this CU for P1 a moment ago).  8 x 8 sub-tiles only: t1 of a 33 x 33 sub-tile would not fit LDS.
// CM: the bottleneck width the kernel is built for, 64 or (the fourth stage of the backbone, Sec. 4: 384 / 96) 96:
// three blocks of 32 mid channels instead of two; conv2's third block is a second pass of the waves that own the
// first; 8 x 8 sub-tiles only.
template <int DT, int C, bool FUSED, int TS, bool PRE, int S = 1, bool PROJ = false, int CO = C, int CM = kCm>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void bottleneck16_kernel(BneckParams p) {
    static_assert(TS == 16 || TS == 8, "output sub-tile side");
    static_assert(CM == 64 || (CM == 96 && TS == 8 && FUSED && !PRE), "the wide form: 8 x 8 sub-tiles, fused, no pre-activation");
    constexpr int NMB = CM / 32;               // blocks of 32 mid channels
    constexpr int KT = CM / 16;                // k-steps over the mid channels (per tap of conv2; of conv3)
    constexpr int NST = 3 * KT;                // stages of P2: tap column x k-step
    constexpr int PS = (CM + 8) * 2;           // LDS bytes per pixel of t1 / t2 (16 B pad); kPS: of a 64-channel chunk of x
    static_assert(S == 1 || (S == 2 && TS == 8 && FUSED && PROJ && !PRE), "the strided form: 8 x 8 sub-tiles, fused, projected");
    static_assert(PROJ || CO == C, "the identity shortcut keeps the channel count");
    constexpr int kBT = TS * S + 3 - S;        // input sub-tile side: TS + 2, or 2 TS + 1 with the stride
    constexpr int kBTPx = kBT * kBT;           // 324 or 100 pixels (289 with the stride)
    constexpr int LOGTS = TS == 16 ? 4 : 3;
    constexpr int RPF = 32 / TS;               // sub-tile rows covered by one 32-pixel MFMA block (2 or 4)
    constexpr int NPB = TS * TS / 32;          // 32-pixel blocks of the output sub-tile (8 or 2)
    constexpr int NP = NPB / 2;                // ... per wave in P2: waves split the rows in two halves (4 or 1)
    constexpr int NF = RPF * (NP - 1) + 3;     // LDS fragments per P2 stage (9 or 3)
    constexpr int W2D = TS == 16 ? (C > 128 ? 3 : 7) : CM == 64 ? 12 : S == 2 ? 3 : 9;   // stages of conv2 weights requested ahead (registers permitting)
    constexpr int W2R = W2D < NST ? W2D : NST; // ... and ring slots holding them
    constexpr int K1 = C / 16;                 // k-steps of conv1
    constexpr int NCH = (C + 63) / 64;         // 64-channel chunks of the input tile (the last may be half empty)
    constexpr int NB3 = CO / 32;               // 32-channel output blocks of conv3
    constexpr int NBW = (NB3 + 3) / 4;         // ... per wave
    constexpr int NBLK1 = (kBTPx + 31) / 32;   // 11 pixel blocks in P1
    constexpr int NBPW1 = (NBLK1 + 3) / 4;     // ... per wave
    constexpr int NVX = (kBTPx * 8 + 255) / 256;   // 16-byte staging vectors per thread and chunk
    static_assert(NVX <= 12, "one vector of the next tile's second chunk is requested per stage of P2");
    constexpr int SB = NBW <= 2 ? NBW : 1;     // channel blocks that leave together through the staging area
    constexpr int NSG = NBW / SB;              // ... groups of them per wave
    constexpr int OPS = SB * 64 + 16;          // LDS bytes per pixel of a group's results (+16 B pad)
    constexpr int CPP = SB * 4;                // 16-byte pieces per pixel of those
    constexpr int PPI = 64 / CPP;              // pixels per wave instruction in the store layout
    constexpr int NI = 64 / PPI;               // instructions per pass (64 pixels)
    constexpr int T1B = kBTPx * PS > 4 * 64 * OPS ? kBTPx * PS : 4 * 64 * OPS;
    constexpr int XSB = kBTPx * kPS > TS * TS * PS ? kBTPx * kPS : TS * TS * PS;
    __shared__ __align__(16) unsigned char t1s[T1B];             // t1; in P3 the four waves' result staging
    __shared__ __align__(16) unsigned char xs[XSB];              // one 64-channel chunk of x in P1, t2 afterwards
    __shared__ __align__(16) uint4 w1s[K1 * NMB * 64];           // conv1 weights, 32x32x16 operand order: [k-step][mid block][lane]
    // 8-pixel sub-tiles serve the launches with few tiles per workgroup, where the time to the first matrix step
    // counts, and their LDS is far from full: conv3's weights are not staged in LDS by the prologue (32 KB of its
    // loads) but read from L2 by each wave for each tile during P2, and (stride 1) conv2's weights live in LDS for
    // the life of the workgroup: 72 KB once instead of 144 KB through registers per tile (two waves share each half).
    constexpr bool kW3FromL2 = TS == 8;
    constexpr bool kW2InLds = TS == 8 && S == 1 && CM == 64;
    __shared__ __align__(16) uint4 w2l[kW2InLds ? 36 * 2 * 64 : 1];     // conv2 weights, [tap][k-step][half][lane]
    __shared__ __align__(16) uint4 w3s[kW3FromL2 ? 1 : NB3 * 4 * 64];   // conv3 weights, [block of 32 outputs][k-step][lane]
    __shared__ __align__(16) float bias_s[2 * CM + CO];         // b1 | b2 | b3 (+ bs): accumulators start from these
    float *pre_s = nullptr;                                      // pre-activation scale | shift
    if constexpr (PRE) {
        __shared__ __align__(16) float pre_store[2 * C];
        pre_s = pre_store;
    }

    const uint16_t *in = (const uint16_t *)p.in;
    uint16_t *out = (uint16_t *)p.out;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: lives in a scalar register
    const int g = lane >> 5, m = lane & 31;
    const int prow = m >> LOGTS, pcol = m & (TS - 1);
    const int rh = wave >> 1, nh = wave & 1;
    const uint32_t per_block = (uint32_t)p.sub_h * p.sub_w;
    const uint32_t G = gridDim.x;
    const uint32_t first = (blockIdx.x & 7) * (G >> 3) + (blockIdx.x >> 3);

    // Addressing convention of this kernel: a wave-uniform 64-bit base plus an unsigned 32-bit per-lane element
    // offset, so that loads and stores use one scalar base and one VGPR instead of a 64-bit VGPR pair per access
    // (36 + 22 + 32 such pairs would otherwise be kept, or spilled, across the tile loop).
    auto decode = [&](uint32_t it) __attribute__((always_inline)) {
        BItem c;
        c.b = fdiv(it, p.div_sub);
        const uint32_t sidx = it - c.b * per_block;
        c.si = (int)fdiv(sidx, p.div_subw);
        c.sj = (int)sidx - c.si * p.sub_w;
        c.n = p.indices[3 * c.b];
        c.by = p.indices[3 * c.b + 1];
        c.bx = p.indices[3 * c.b + 2];
        return c;
    };

    const int nact_raw = *p.count;
    BItem cur = decode(min(first, (uint32_t)p.cap * per_block - 1u));
    const int nact = max(min(nact_raw, p.cap), 0);
    const uint32_t items = (uint32_t)nact * per_block;
    bool use16 = false;
    if (p.per16 > 0) {
        const unsigned long long r16 = ((unsigned long long)nact * p.per16 + 255u) >> 8, r8 = ((unsigned long long)nact * p.per8 + 255u) >> 8;
        use16 = r16 * 8u <= r8 * (unsigned long long)p.cost8;
    }
    if (first >= items || use16 != (p.want16 != 0)) return;

    // ---- geometry of a sub-tile: origin in memory and the rows / columns that exist and lie inside the image
    struct TileGeo {
        __amdgpu_buffer_rsrc_t xrs;     // the sample (fused) or tile that holds the sub-tile
        uint32_t xorg;                  // byte offset of the sub-tile's pixel (0, 0) in it; wraps below zero above / left of the image
        int gx0;                        // image column of sub-tile column 0 (on tiles: tile column)
        int rlo, rhi, clo, chi, ty0, tx0;
    };
    const int in_w = FUSED ? p.W : p.tw;                                  // pixels per row of the addressed array
    const int row_stride = in_w * C;                                      // elements between rows of the input
    const uint32_t in_bytes = (uint32_t)(FUSED ? p.H : p.th) * row_stride * 2u;
    auto geometry_of = [&](const BItem &c) __attribute__((always_inline)) {
        TileGeo t;
        t.ty0 = c.si * TS;                                                    // sub-tile origin inside the OUTPUT block
        t.tx0 = c.sj * TS;
        const int iy0 = t.ty0 * S, ix0 = t.tx0 * S;                           // ... and inside the input tile
        const int gy0 = p.g_in.boffset_h + c.by * p.g_in.bstride_h + iy0;     // sub-tile origin in image coordinates
        const int gx0 = p.g_in.boffset_w + c.bx * p.g_in.bstride_w + ix0;
        t.rlo = max(0, -gy0);
        t.rhi = min(min(kBT, p.th - iy0), p.H - gy0);
        t.clo = max(0, -gx0);
        t.chi = min(min(kBT, p.tw - ix0), p.W - gx0);
        const uint16_t *base = FUSED ? in + (long long)c.n * p.H * row_stride : in + (long long)c.b * p.th * row_stride;
        const int y0 = FUSED ? gy0 : iy0, x0 = FUSED ? gx0 : ix0;
        t.xrs = __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, (int)in_bytes, (int)kBufWord3B);
        t.xorg = (uint32_t)(y0 * row_stride + x0 * C) * 2u;
        t.gx0 = x0;
        return t;
    };

    // ---- staging of one 64-channel chunk: vector v = tid + 256 k covers pixel v / 8, channels (v % 8) * 8 .. + 8.
    //      Eight neighbouring lanes read one pixel's 128 contiguous bytes, so a wave instruction touches 8 full
    //      cache lines.  Offsets are recomputed per use: keeping them would cost 2 registers per vector.
    uint4 sx0[NVX], sx1[NVX];                                             // two chunks in flight (slot 0 / slot 1)
    // The vectors of a chunk are requested in order through an iterator that holds the pixel's column in the
    // sub-tile and its byte offset: from vector k to k + 1 the pixel index grows by 32, i.e. by 32 / kBT rows and
    // 32 % kBT columns with at most one carry (a division per vector cost twice the vector instructions).
    struct VecIt { int col; uint32_t off; };
    auto vec_begin = [&](const TileGeo &t, int chunk) __attribute__((always_inline)) {
        int tid = (int)threadIdx.x;
        asm volatile("" : "+v"(tid));     // opaque: otherwise the per-vector offsets are hoisted out of the tile loop and spilled
        const int p0 = tid >> 3, c8 = tid & 7;
        const int row = p0 / kBT;
        VecIt it;
        it.col = p0 - row * kBT;
        it.off = t.xorg + (uint32_t)(row * row_stride + it.col * C + c8 * 8 + chunk * 64) * 2u;
        return it;
    };
    // vector k of the chunk (k in order from 0; live = false: a tile that does not exist, nothing is read)
    auto fetch_vec = [&](const TileGeo &t, int chunk, auto slot_tag, int k, bool live, VecIt &it) __attribute__((always_inline)) {
        constexpr int slot = decltype(slot_tag)::value;
        // rows outside the image are outside the descriptor; columns outside would wrap into the neighbouring
        // row, so they (and the unused tail of the last vector) get the out-of-range offset: zeros either way
        bool ok = live && (uint32_t)(t.gx0 + it.col) < (uint32_t)in_w;
        if (C % 64 != 0) ok = ok && ((int)(threadIdx.x & 7) * 8 + chunk * 64 < C);
        if ((k + 1) * 256 > kBTPx * 8) ok = ok && (int)threadIdx.x < kBTPx * 8 - k * 256;
        const uint4 val = bload16(t.xrs, ok ? it.off : kOutOfRangeB);
        if (slot == 0) sx0[k] = val;
        else sx1[k] = val;
        constexpr int RA = 32 / kBT, CA = 32 % kBT;
        const int col = it.col + CA;
        const bool carry = col >= kBT;
        it.col = carry ? col - kBT : col;
        it.off += (uint32_t)(RA * row_stride + CA * C) * 2u + (carry ? (uint32_t)(row_stride - kBT * C) * 2u : 0u);
    };
    auto fetch_chunk = [&](const TileGeo &t, int chunk, auto slot_tag) __attribute__((always_inline)) {
        VecIt it = vec_begin(t, chunk);
#pragma unroll
        for (int k = 0; k < NVX; ++k) fetch_vec(t, chunk, slot_tag, k, true, it);
        __builtin_amdgcn_sched_barrier(0);                                // all loads issued here, in this order
    };
    // With a pre-activation the chunk is transformed on its way to LDS: conv1 reads ReLU(scale * x + shift), the
    // residual (requested separately) stays x.  A thread's vectors all hold the same eight channels of the chunk.
    auto stash_chunk = [&](auto slot_tag, int chunk) __attribute__((always_inline)) {
        constexpr int slot = decltype(slot_tag)::value;
        if constexpr (!PRE) {
#pragma unroll
            for (int k = 0; k < NVX; ++k) {
                const int v = (int)threadIdx.x + k * 256;
                // the tail beyond the last pixel goes to the 16 pad bytes of the last pixel: no branch
                const int dst = v < kBTPx * 8 ? (v >> 3) * kPS + (v & 7) * 16 : (kBTPx - 1) * kPS + kCm * 2;
                *(uint4 *)(xs + dst) = slot == 0 ? sx0[k] : sx1[k];
            }
        } else {
            const int c0 = chunk * 64 + ((int)threadIdx.x & 7) * 8;
            const float4 a0 = *(const float4 *)(pre_s + c0), a1 = *(const float4 *)(pre_s + c0 + 4);
            const float4 h0 = *(const float4 *)(pre_s + C + c0), h1 = *(const float4 *)(pre_s + C + c0 + 4);
            const float sc[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
            const float sh[8] = {h0.x, h0.y, h0.z, h0.w, h1.x, h1.y, h1.z, h1.w};
#pragma unroll
            for (int k = 0; k < NVX; ++k) {
                const int v = (int)threadIdx.x + k * 256;
                const int dst = v < kBTPx * 8 ? (v >> 3) * kPS + (v & 7) * 16 : (kBTPx - 1) * kPS + kCm * 2;
                const uint4 val = slot == 0 ? sx0[k] : sx1[k];
                uint32_t w[4] = {val.x, val.y, val.z, val.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float lo = fmaf(sc[2 * i], unpack_lo<DT>(w[i]), sh[2 * i]);
                    const float hi = fmaf(sc[2 * i + 1], unpack_hi<DT>(w[i]), sh[2 * i + 1]);
                    w[i] = pack2<DT>(__int_as_float(relu_bits(lo)), __int_as_float(relu_bits(hi)));
                }
                *(uint4 *)(xs + dst) = make_uint4(w[0], w[1], w[2], w[3]);
            }
        }
    };

    // ---- Prologue.  What does not depend on the block list is requested first and arrives while the list's entry
    //      does: W1 (and W3) for LDS and the biases (all loads before all LDS stores); then the first two chunks of
    //      the first tile are requested.
    using Slot0 = std::integral_constant<int, 0>;
    using Slot1 = std::integral_constant<int, 1>;
    const uint4 *w3g = (const uint4 *)p.w3 + p.w3_off;           // [ng][ks][nb][lane] -> [ng*2+nb][ks][lane]
    TileGeo geo;
    {
        const uint4 *w1g = (const uint4 *)p.w1 + p.w1_off;       // [ks][nb][lane], one group of 64 outputs
        static_assert(K1 * NMB * 64 % 256 == 0, "conv1's weights divide among the threads");
        constexpr int N1 = K1 * NMB * 64 / 256, N3 = kW3FromL2 ? 0 : NB3 * 4 * 64 / 256, NBI = (2 * CM + CO + 255) / 256;
        constexpr int N2 = kW2InLds ? 36 * 2 * 64 / 256 : 0;
        uint4 t1v[N1], t3v[N3 > 0 ? N3 : 1], t2v[N2 > 0 ? N2 : 1];
        float bv[NBI];
#pragma unroll
        for (int k = 0; k < N1; ++k) {       // (by value: a struct copy kept the array in memory)
            const int i = threadIdx.x + k * 256;
            const int ln = i & 63, q = i >> 6, mb = q % NMB, ks = q / NMB;     // packed: [group of 64][k-step][block of 32][lane]
            t1v[k] = gload16((gvec_t)w1g + ((((mb >> 1) * K1 + ks) * 2 + (mb & 1)) * 64 + ln));
        }
#pragma unroll
        for (int k = 0; k < N3; ++k) {
            const int i = threadIdx.x + k * 256;
            const int ln = i & 63, ks = (i >> 6) & 3, nbg = i >> 8;
            // (k-steps the packed copy does not hold multiply zeros of t2: any finite fragment will do)
            t3v[k] = gload16((gvec_t)w3g + ((((size_t)(nbg >> 1) * p.km + min(ks, p.km - 1)) * 2 + (nbg & 1)) * 64 + ln));
        }
#pragma unroll
        for (int k = 0; k < N2; ++k) {
            const int i = threadIdx.x + k * 256;
            const int ln = i & 63, half = (i >> 6) & 1, kc = (i >> 7) & 3, tap = i >> 9;
            t2v[k] = gload16((gvec_t)((const uint4 *)p.w2 + p.w2_off) + ((tap * p.km + min(kc, p.km - 1)) * 128 + half * 64 + ln));
        }
        // biases b1 | b2 | b3 (+ bs), zero beyond the unit's width: every lane loads from a clamped address (a load
        // under a condition is waited for at once)
#pragma unroll
        for (int k = 0; k < NBI; ++k) {
            const int i = threadIdx.x + k * 256;
            const int i3 = min(max(i - 2 * CM, 0), CO - 1);
            const float *src = i < CM ? p.b1 + min(i, p.Cm - 1) : i < 2 * CM ? p.b2 + min(i - CM, p.Cm - 1) : p.b3 + i3;
            float v = *src;
            if (PROJ) v += i >= 2 * CM ? p.bs[i3] : 0.f;
            bv[k] = (i < 2 * CM && (i < CM ? i : i - CM) >= p.Cm) ? 0.f : v;
        }
        geo = geometry_of(cur);
        fetch_chunk(geo, 0, Slot0{});
        if (NCH > 1) fetch_chunk(geo, 1, Slot1{});
#pragma unroll
        for (int k = 0; k < N1; ++k) w1s[threadIdx.x + k * 256] = t1v[k];
#pragma unroll
        for (int k = 0; k < N3; ++k) w3s[threadIdx.x + k * 256] = t3v[k];
#pragma unroll
        for (int k = 0; k < N2; ++k) w2l[threadIdx.x + k * 256] = t2v[k];
#pragma unroll
        for (int k = 0; k < NBI; ++k)
            if ((int)threadIdx.x + k * 256 < 2 * CM + CO) bias_s[threadIdx.x + k * 256] = bv[k];
        if constexpr (PRE)
            for (int i = threadIdx.x; i < 2 * C; i += 256) pre_s[i] = i < C ? p.pre_scale[i] : p.pre_shift[i - C];
    }
    // 16 consecutive biases from LDS as an accumulator-shaped vector
    auto load_bias16 = [&](int i0) __attribute__((always_inline)) {
        f32x16b v;
        const float4 q0 = *(const float4 *)(bias_s + i0), q1 = *(const float4 *)(bias_s + i0 + 4);
        const float4 q2 = *(const float4 *)(bias_s + i0 + 8), q3 = *(const float4 *)(bias_s + i0 + 12);
        v[0] = q0.x; v[1] = q0.y; v[2] = q0.z; v[3] = q0.w; v[4] = q1.x; v[5] = q1.y; v[6] = q1.z; v[7] = q1.w;
        v[8] = q2.x; v[9] = q2.y; v[10] = q2.z; v[11] = q2.w; v[12] = q3.x; v[13] = q3.y; v[14] = q3.z; v[15] = q3.w;
        return v;
    };
    __syncthreads();                                 // weights and biases visible to every wave

    for (uint32_t it = first; it < items; it += G) {
        // Where conv2's weights do not live in LDS (16-pixel sub-tiles, the strided and the wide form) they are re-read
        // from L2 for every tile, three fragments per stage of P2 for this wave's 32 output channels, through a ring of
        // W2R stages, W2D stages requested ahead (holding all 36 fragments would cost 144 registers that the residual
        // needs; 8-pixel sub-tiles of the strided form, whose stages are short, hold them all).
        uint4 w2s[W2R][3];
        const uint4 *w2p = (const uint4 *)p.w2 + p.w2_off;                        // wave-uniform
        asm volatile("" : "+s"(w2p));      // opaque per iteration: keeps the loads inside the tile loop
        // stage st of mid block cb: packed [group of 64 outputs][tap][k-step][block of 32][lane]
        auto fetch_w2 = [&](int st, int cb) __attribute__((always_inline)) {
            const uint4 *wb = w2p + ((size_t)(cb >> 1) * 9 * p.km * 2 + (cb & 1)) * 64;
#pragma unroll
            for (int r = 0; r < 3; ++r)     // (as for W3: a k-step beyond km multiplies zeros of t1)
                w2s[st % W2R][r] = gload16((gvec_t)wb + ((r * 3 + st / KT) * p.km + min(st % KT, p.km - 1)) * 128 + (uint32_t)lane);
        };

        // ---- where this tile's results go and, for the fused form, where the residual x comes from.  Layout of
        //      P3's memory accesses: instruction i of a pass (64 pixels = pixel blocks 2bp, 2bp+1) covers pixels
        //      i*PPI + lane/CPP of the pass, 16-byte piece lane%CPP of the wave's channels.
        const int out_w = FUSED ? p.Wo : p.ow;
        __amdgpu_buffer_rsrc_t yrs;
        uint32_t yorg;                   // byte offset of the sub-tile's output pixel (0, 0), first channel of the wave
        int ox;                          // image column of sub-tile column 0 (on tiles: block column)
        {
            uint16_t *ybase = out;
            int oy;
            if (FUSED) {
                oy = p.g_out.boffset_h + cur.by * p.g_out.bstride_h + geo.ty0;
                ox = p.g_out.boffset_w + cur.bx * p.g_out.bstride_w + geo.tx0;
                ybase += (long long)cur.n * p.Ho * p.Wo * CO;
            } else {
                oy = geo.ty0;
                ox = geo.tx0;
                ybase += (long long)cur.b * p.oh * p.ow * CO;
            }
            const uint32_t ybytes = (uint32_t)(FUSED ? p.Ho : p.oh) * out_w * CO * 2u;
            yrs = __builtin_amdgcn_make_buffer_rsrc((void *)ybase, 0, (int)ybytes, (int)kBufWord3B);
            yorg = (uint32_t)((oy * out_w + ox) * CO + wave * NBW * 32) * 2u;
        }
        // Rows below the image are outside the descriptors by themselves; columns outside and (C = 64) the channel
        // blocks of waves without work get the out-of-range offset.
        // Pixel q = i * PPI + lane / CPP of the pass: its row is a constant of (bp, i) plus (8-pixel sub-tiles with
        // 16 pixels per instruction) a lane part, its column one of at most two lane parts.  The lane parts are kept
        // (one or two registers), the row constant is added per access from a scalar.
        constexpr int NCOLV = (TS == 16 && PPI == 8) ? 2 : 1;
        uint32_t lane_off[NCOLV];
        const uint32_t out_row_bytes = (uint32_t)(out_w * CO) * 2u;
        // (computed where first needed, P3, or P1 with a pre-activation: kept across P2 they were spilled)
        auto set_lane_off = [&]() __attribute__((always_inline)) {
            const int l = lane / CPP;
            const int rowl = (TS == 8 && PPI == 16) ? (l >> 3) : 0;
#pragma unroll
            for (int v = 0; v < NCOLV; ++v) {
                const int col = NCOLV == 2 ? v * 8 + l : (l & (TS - 1));
                const bool ok = wave * NBW < NB3 && (uint32_t)(ox + col) < (uint32_t)out_w;
                lane_off[v] = ok ? yorg + (uint32_t)((rowl * out_w + col) * CO) * 2u + (lane % CPP) * 16 : kOutOfRangeB;
            }
        };
        if (PRE) set_lane_off();
        auto out_offset = [&](int bp, int i) __attribute__((always_inline)) {
            const int rowc = RPF * (2 * bp + ((i * PPI) >> 5)) + (((i * PPI) & 31) >> LOGTS);
            // (an out-of-range lane part stays out of range: the sum is below 2^32)
            return lane_off[NCOLV == 2 ? (i & 1) : 0] + (uint32_t)rowc * out_row_bytes;
        };
        // residual x of the block with a pre-activation (the LDS copy of x is the transformed one): read again, in the
        // store layout, in the middle of P1, when half of the tile's chunks have just come through L2 and the other
        // half is about to, so that each of its cache lines crosses the memory fabric once.  (Requested after P1, half
        // of the block had been evicted again: L2 holds about 3 microseconds of this kernel's traffic.)
        constexpr int NPASS = NPB / 2;
        uint4 rres[NPASS][NI];                   // pre-activation form: x in the store layout
        uint4 rb[NPASS][2][NBW][2];              // otherwise: x as MFMA B operands (see below)
        auto fetch_residual = [&](int bp0, int bp1) __attribute__((always_inline)) {
            if (!FUSED || PROJ || !PRE) return;
#pragma unroll
            for (int bp = bp0; bp < bp1; ++bp)
#pragma unroll
                for (int i = 0; i < NI; ++i) rres[bp][i] = bload16(geo.xrs, out_offset(bp, i));     // x and y have one shape
            __builtin_amdgcn_sched_barrier(0);
        };
        // Without a pre-activation the residual never leaves the chip: the wave's output channels are (part of) one
        // 64-channel chunk of the input, which lies in LDS for a while during P1.  The wave copies the block's pixels
        // of it to registers then, as B operands (lane (g, m): pixel m of a block of 32, eight channels), and P3 adds
        // them to its accumulators with two more matrix steps per block against a 0/1 matrix: the sum x + t3 is formed
        // in fp32 and rounded once, and the vector unit, which bounds P3, has nothing to do for it.
        constexpr bool kResidualFromLds = FUSED && !PROJ && !PRE;
        // (block j of the wave = block wave * NBW + j of the unit's channels: half of chunk (wave * NBW + j) / 2)
        auto residual_from_lds = [&](int j) __attribute__((always_inline)) {
            const int roff = (((wave * NBW + j) & 1) * 32 + g * 8) * 2;
#pragma unroll
            for (int bp = 0; bp < NPASS; ++bp)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int q = (2 * bp + u) * 32 + m;                       // output pixel of the sub-tile
                    const unsigned char *src = xs + (((q >> LOGTS) + 1) * kBT + (q & (TS - 1)) + 1) * kPS + roff;
#pragma unroll
                    for (int k2 = 0; k2 < 2; ++k2) rb[bp][u][j][k2] = *(const uint4 *)(src + (k2 * 16) * 2);
                }
        };

        const uint32_t nit = it + G;                                      // the workgroup's next tile, if any
        const bool has_next = nit < items;
        BItem nxt = cur;
        TileGeo ngeo = geo;

        // ================= P1: t1 = ReLU(W1 x + b1), zero outside the image =================
        // x passes through LDS in 64-channel chunks: coalesced global loads -> registers -> xs -> MFMA B operands.
        // Wave w owns pixel blocks w, w+4, w+8 (32 pixels each, row-major over the input sub-tile) and all mid channels.
        {
            f32x16b acc[NBPW1][NMB];
#pragma unroll
            for (int j = 0; j < NBPW1; ++j)
#pragma unroll
                for (int mb = 0; mb < NMB; ++mb) acc[j][mb] = load_bias16(mb * 32 + g * 16);
            int boff[NBPW1];                                             // LDS byte offset of this lane's pixel
#pragma unroll
            for (int j = 0; j < NBPW1; ++j) boff[j] = min((wave + 4 * j) * 32 + m, kBTPx - 1) * kPS + g * 16;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                if (c & 1) stash_chunk(Slot1{}, c);
                else stash_chunk(Slot0{}, c);
                __syncthreads();                                         // chunk c visible
                if (c + 2 < NCH) {
                    if (c & 1) fetch_chunk(geo, c + 2, Slot1{});
                    else fetch_chunk(geo, c + 2, Slot0{});
                }
                if (c == (NCH > 1 ? 1 : 0)) fetch_residual(0, NPASS);
                if (c == NCH - 1) {
                    // Both staging slots are free from here on.  The next tile's first two chunks are requested a vector
                    // of each per stage of P2, which leaves the memory pipeline idle otherwise.  Measured: a load costs
                    // the wave about 100 clocks there, 450 among the stores of P3, and 200 in one burst of 22 after P2;
                    // while t1 is written (the end of P1) they cost the same as in P2 but their registers, on top of
                    // the accumulators of P1, made the compiler spill, and a spill's reload waits for every load in flight.
                    nxt = decode(min(nit, (uint32_t)p.cap * per_block - 1u));
                    ngeo = geometry_of(nxt);
                }
                if (kResidualFromLds) {
#pragma unroll
                    for (int j = 0; j < NBW; ++j)
                        if (c == min((wave * NBW + j) >> 1, NCH - 1)) residual_from_lds(j);
                }
                // fragments of k-step k4+1 are read from LDS while the MFMAs of k-step k4 run
                uint4 af[2][NMB], bf[2][NBPW1];
#pragma unroll
                for (int mb = 0; mb < NMB; ++mb) af[0][mb] = w1s[((c * 4) * NMB + mb) * 64 + lane];
#pragma unroll
                for (int j = 0; j < NBPW1; ++j) bf[0][j] = *(const uint4 *)(xs + boff[j]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int k4 = 0; k4 < 4 && c * 4 + k4 < K1; ++k4) {       // the last chunk of C = 96 holds two k-steps
                    if (k4 + 1 < 4 && c * 4 + k4 + 1 < K1) {
#pragma unroll
                        for (int mb = 0; mb < NMB; ++mb) af[(k4 + 1) & 1][mb] = w1s[((c * 4 + k4 + 1) * NMB + mb) * 64 + lane];
#pragma unroll
                        for (int j = 0; j < NBPW1; ++j) bf[(k4 + 1) & 1][j] = *(const uint4 *)(xs + boff[j] + (k4 + 1) * 32);
                    }
#pragma unroll
                    for (int j = 0; j < NBPW1; ++j) {
                        // (wave 3's third block does not exist: it recomputes pixel 323 and the result is dropped;
                        //  a branch here would cost a copy of every accumulator per step)
#pragma unroll
                        for (int mb = 0; mb < NMB; ++mb) acc[j][mb] = mfma32<DT>(af[k4 & 1][mb], bf[k4 & 1][j], acc[j][mb]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (c + 1 < NCH) __syncthreads();                        // everyone done with xs before the next chunk
            }
            // the first stages of conv2's weights come from L2 while t1 is written (requested only now: no input chunk of
            // this tile is queued behind them, and their registers are not held through the last chunk's matrix steps)
            if (!kW2InLds) {
#pragma unroll
                for (int st = 0; st < W2R; ++st) fetch_w2(st, nh);
            }
#pragma unroll
            for (int j = 0; j < NBPW1; ++j) {
                // lanes past the last pixel were fed pixel 323's operands: they write pixel 323's values again
                const int pi = min((wave + 4 * j) * 32 + m, kBTPx - 1);
                const int row = pi / kBT, col = pi - row * kBT;
                const bool inside = row >= geo.rlo && row < geo.rhi && col >= geo.clo && col < geo.chi;
                const uint32_t keep = inside ? 0xffffffffu : 0u;         // (a mask, not a select: selects became branches here)
#pragma unroll
                for (int mb = 0; mb < NMB; ++mb) {
                    uint32_t w[8];
#pragma unroll
                    for (int k = 0; k < 8; ++k) w[k] = relu_pack2<DT>(acc[j][mb][2 * k], acc[j][mb][2 * k + 1]) & keep;
                    uint4 *d = (uint4 *)(t1s + pi * PS + mb * 64 + g * 32);     // channels mb * 32 + g * 16 .. + 16
                    d[0] = make_uint4(w[0], w[1], w[2], w[3]);
                    d[1] = make_uint4(w[4], w[5], w[6], w[7]);
                }
            }
        }
        __syncthreads();

        // ================= P2: t2 = ReLU(W2 * t1 + b2) -> xs =================
        uint4 w3r[KT][NBW];                                              // conv3's weights of this wave's channels
        if constexpr (kW3FromL2) {
#pragma unroll
            for (int j = 0; j < NBW; ++j) {
                const int nbg = min(wave * NBW + j, NB3 - 1);
#pragma unroll
                for (int ks = 0; ks < KT; ++ks)
                    w3r[ks][j] = w3g[(((size_t)(nbg >> 1) * p.km + min(ks, p.km - 1)) * 2 + (nbg & 1)) * 64 + lane];
            }
        }
        // wave (rh, nh): output rows rh*TS/2 .. + TS/2 (NP pixel blocks of RPF rows), mid channels nh*32 .. + 32; with
        // three blocks of mid channels the waves nh = 0 then take the third in a second pass.
        // Fragment j of a stage holds input rows rh*TS/2 + j .. + RPF at tap column t; pixel block P with tap row r
        // reads fragment RPF*P + r.
#pragma unroll
        for (int pass = 0; pass < (NMB > 2 ? 2 : 1); ++pass) {
            const int cb = pass == 0 ? nh : 2;                            // block of 32 mid channels, wave-uniform
            if (pass == 1) {
                if (nh != 0) continue;
#pragma unroll
                for (int st = 0; st < W2R; ++st) fetch_w2(st, cb);
            }
            const int cm0 = cb * 32 + g * 16;                             // this lane's 16 mid channels
            f32x16b acc[NP];
            const f32x16b bias2 = load_bias16(CM + cm0);
            const unsigned char *L = t1s + ((rh * (TS / 2) + prow) * S * kBT + pcol * S) * PS + g * 16;
            // One set of fragments: a fragment is re-read for the next stage right after the last matrix step of this
            // stage that takes it (the matrix unit has read its operands by then, the LDS answer comes later still);
            // its next use is at least four matrix steps away.  (Two sets cost 36 registers more; the phase is the
            // kernel's register peak.)
            uint4 xf[NF], wl[2][3];
            // (kW2InLds) fragment r of stage st: tap (r, st / 4), k-step st % 4, this wave's half of the mid channels
            const uint4 *wlp = w2l + nh * 64 + lane;
            VecIt nit0 = vec_begin(ngeo, 0), nit1 = vec_begin(ngeo, NCH > 1 ? 1 : 0);
            static_assert(S == 1 || NF == 3, "with a stride a pixel block's three tap rows are three fragments of their own");
#pragma unroll
            for (int j = 0; j < NF; ++j) xf[j] = *(const uint4 *)(L + (j * kBT) * PS);
            if (kW2InLds) {
#pragma unroll
                for (int r = 0; r < 3; ++r) wl[0][r] = wlp[(r * 3 * 4) * 128];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int st = 0; st < NST; ++st) {
                const int tn = (st + 1) / KT, kcn = (st + 1) % KT;
#pragma unroll
                for (int mm = 0; mm < 3 * NP; ++mm) {
                    const int r = mm / NP, P = mm % NP;
                    constexpr int kNoReload = -1;
                    acc[P] = mfma32<DT>(kW2InLds ? wl[st & 1][r] : w2s[st % W2R][r], xf[RPF * P + r], (st == 0 && r == 0) ? bias2 : acc[P]);
                    // fragment f = RPF * P + r also serves (r + RPF, P - 1), later in the stage, if that tap row exists
                    const int f = RPF * P + r;
                    const bool last_use = !(r + RPF <= 2 && P >= 1);
                    const int reload = last_use && st + 1 < NST ? f : kNoReload;
                    if (kW2InLds && mm < 3 && st + 1 < NST) wl[(st + 1) & 1][mm] = wlp[((mm * 3 + tn) * 4 + kcn) * 128];
                    if (pass == 0 && mm == 0 && st < NVX) fetch_vec(ngeo, 0, Slot0{}, st, has_next, nit0);
                    if (NCH > 1 && pass == 0 && mm == 1 && st < NVX) fetch_vec(ngeo, 1, Slot1{}, st, has_next, nit1);
                    if (reload != kNoReload) xf[reload] = *(const uint4 *)(L + (reload * kBT + tn) * PS + kcn * 32);
                    if (!kW2InLds && mm == 3 * NP - 1 && st + W2D < NST) fetch_w2(st + W2D, cb);       // into the slot this stage just freed
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
#pragma unroll
            for (int P = 0; P < NP; ++P) {
                const int po = (rh * (TS / 2) + RPF * P + prow) * TS + pcol;
                uint32_t w[8];
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    w[k] = relu_pack2<DT>(acc[P][2 * k], acc[P][2 * k + 1]);
                uint4 *d = (uint4 *)(xs + po * PS + cm0 * 2);
                d[0] = make_uint4(w[0], w[1], w[2], w[3]);
                d[1] = make_uint4(w[4], w[5], w[6], w[7]);
            }
        }
        __syncthreads();

        // ================= P3: t3 = W3 t2 + b3 (+ x), two pixel blocks (64 pixels) per pass =================
        {
            if constexpr (!kW3FromL2) {
#pragma unroll
                for (int j = 0; j < NBW; ++j) {
                    const int nbg = min(wave * NBW + j, NB3 - 1);         // this wave's neighbouring blocks of 32 channels
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks) w3r[ks][j] = w3s[(nbg * 4 + ks) * 64 + lane];     // (this form: KT = 4)
                }
            }
            unsigned char *ost = t1s + wave * (64 * OPS);                 // t1 is dead: the wave's private staging area
            if (!PRE) set_lane_off();
            // P3 is bound by LDS traffic, and accumulators that start from the bias read it from LDS in every pass (16
            // of a pass's 40 LDS instructions; kept in registers it would take 32 of them).  The bias is added by the
            // matrix unit instead: split into three bf16 / f16 pieces (b = p0 + p1 + p2 exactly for bf16: 3 x 8 bits
            // cover fp32's 24; f16 drops what lies below its smallest number, under 1e-7), as columns 0..2 of an A
            // operand whose B operand is all ones in those rows: one more matrix step per block and pass, no LDS.
            uint4 biasA[NBW], onesB;
            {
                const int ol = ((m >> 2) & 1) * 16 + (m >> 3) * 4 + (m & 3);      // channel of A row m within its block
                const uint32_t one = DT == SBNET_BF16 ? 0x3F80u : 0x3C00u;
                onesB = g == 0 ? make_uint4(one | one << 16, one, 0u, 0u) : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
                for (int j = 0; j < NBW; ++j) {
                    const float b = bias_s[2 * CM + min(wave * NBW + j, NB3 - 1) * 32 + ol];
                    const uint32_t w0 = pack2<DT>(b, 0.f);
                    const float r1 = b - unpack_lo<DT>(w0);
                    const uint32_t w1 = pack2<DT>(r1, 0.f);
                    const float r2 = r1 - unpack_lo<DT>(w1);
                    const uint32_t w2 = pack2<DT>(r2, 0.f);
                    biasA[j] = g == 0 ? make_uint4((w0 & 0xffffu) | w1 << 16, w2 & 0xffffu, 0u, 0u) : make_uint4(0u, 0u, 0u, 0u);
                }
            }
            const f32x16b zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            // Blocks of 32 pixels per pass: two for waves with one block of channels (two independent chains of matrix
            // steps), one for waves with two (half the accumulators and operands: registers are short in P3)
            constexpr int UB = NBW >= 2 ? 1 : 2;
            static_assert(NI % 2 == 0, "a pass's store instructions split between its two pixel blocks");
            // 0/1 matrix that routes channel k of the residual operand to the accumulator row holding that channel
            // (rows are permuted as the packed weights are: row rho holds channel (rho/4 % 2) * 16 + rho/8 * 4 + rho % 4)
            uint4 ida[2];
            if constexpr (kResidualFromLds) {
                const int ol = ((m >> 2) & 1) * 16 + (m >> 3) * 4 + (m & 3);
                const uint32_t one = DT == SBNET_BF16 ? 0x3F80u : 0x3C00u;
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2) {
                    const int t = ol - k2 * 16 - g * 8;                       // this lane's element that is 1, if in 0..7
                    const uint32_t w = (t & 1) ? one << 16 : one;
                    ida[k2] = make_uint4((t >> 1) == 0 ? w : 0u, (t >> 1) == 1 ? w : 0u, (t >> 1) == 2 ? w : 0u, (t >> 1) == 3 ? w : 0u);
                }
            }
#pragma unroll
            for (int bp = 0; bp < NPASS; ++bp)
#pragma unroll
            for (int u0 = 0; u0 < 2; u0 += UB) {
                uint4 tf[2][KT];
#pragma unroll
                for (int u = u0; u < u0 + UB; ++u)
#pragma unroll
                    for (int ks = 0; ks < KT; ++ks)
                        tf[u][ks] = *(const uint4 *)(xs + ((2 * bp + u) * 32 + m) * PS + ks * 32 + g * 16);
                f32x16b acc[2][NBW];
#pragma unroll
                for (int u = u0; u < u0 + UB; ++u)
#pragma unroll
                    for (int j = 0; j < NBW; ++j) acc[u][j] = mfma32<DT>(biasA[j], onesB, zero16);
#pragma unroll
                for (int ks = 0; ks < KT; ++ks)
#pragma unroll
                    for (int u = u0; u < u0 + UB; ++u)
#pragma unroll
                        for (int j = 0; j < NBW; ++j) acc[u][j] = mfma32<DT>(w3r[ks][j], tf[u][ks], acc[u][j]);
                if constexpr (kResidualFromLds) {
#pragma unroll
                    for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
                        for (int u = u0; u < u0 + UB; ++u)
#pragma unroll
                            for (int j = 0; j < NBW; ++j) acc[u][j] = mfma32<DT>(ida[k2], rb[bp][u][j][k2], acc[u][j]);
                }
                if constexpr (PROJ) {
                    // the shortcut: + Ws x at the input pixels under the pass's 64 output pixels, K = C in steps of 16,
                    // four k-steps of loads in flight (operands straight from L2, 16 bytes per lane)
                    const uint4 *wsg = (const uint4 *)p.ws + p.ws_off;            // [ng][ks][nb][lane]
                    uint32_t xoff[2];
#pragma unroll
                    for (int u = u0; u < u0 + UB; ++u) {
                        const int q = (2 * bp + u) * 32 + m;                          // output pixel of the sub-tile
                        const int orow = q >> LOGTS, ocol = q & (TS - 1);
                        xoff[u] = geo.xorg + (uint32_t)((orow * S + 1) * row_stride + (ocol * S + 1) * C + g * 8) * 2u;
                    }
                    constexpr int KB = 4;
#pragma unroll
                    for (int k0 = 0; k0 < K1; k0 += KB) {
                        uint4 xb[KB][2], wa[KB][NBW];
#pragma unroll
                        for (int kk = 0; kk < KB; ++kk) {
                            if (k0 + kk >= K1) continue;
#pragma unroll
                            for (int u = u0; u < u0 + UB; ++u) xb[kk][u] = bload16(geo.xrs, xoff[u] + (uint32_t)(k0 + kk) * 32u);
#pragma unroll
                            for (int j = 0; j < NBW; ++j) {
                                const int nbg = min(wave * NBW + j, NB3 - 1);
                                wa[kk][j] = wsg[(((size_t)(nbg >> 1) * K1 + (k0 + kk)) * 2 + (nbg & 1)) * 64 + lane];
                            }
                        }
#pragma unroll
                        for (int kk = 0; kk < KB; ++kk) {
                            if (k0 + kk >= K1) continue;
#pragma unroll
                            for (int u = u0; u < u0 + UB; ++u)
#pragma unroll
                                for (int j = 0; j < NBW; ++j) acc[u][j] = mfma32<DT>(wa[kk][j], xb[kk][u], acc[u][j]);
                        }
                    }
                }
                // MFMA layout -> LDS: lane (g, m) holds channels j*32 + g*16 .. + 16 of pixel u*32 + m; SB blocks of
                // channels go through the staging area together (waves with three blocks: one at a time)
#pragma unroll
                for (int sg = 0; sg < NSG; ++sg) {
#pragma unroll
                    for (int u = u0; u < u0 + UB; ++u)
#pragma unroll
                        for (int jj = 0; jj < SB; ++jj) {
                            const int j = sg * SB + jj;
                            uint32_t w[8];
#pragma unroll
                            for (int k = 0; k < 8; ++k) w[k] = pack2<DT>(acc[u][j][2 * k], acc[u][j][2 * k + 1]);
                            uint4 *d = (uint4 *)(ost + (u * 32 + m) * OPS + jj * 64 + g * 32);
                            d[0] = make_uint4(w[0], w[1], w[2], w[3]);
                            d[1] = make_uint4(w[4], w[5], w[6], w[7]);
                        }
                    // LDS -> store layout (LDS serves one wave's accesses in order: no wait between the two), add, store
#pragma unroll
                    for (int i = u0 * (NI / 2); i < (u0 + UB) * (NI / 2); ++i) {
                        uint4 v = *(const uint4 *)(ost + (i * PPI + lane / CPP) * OPS + (lane % CPP) * 16);
                        if (FUSED && !PROJ && PRE) {
                            const uint4 rv = rres[bp][i];
                            v.x = pack2<DT>(unpack_lo<DT>(v.x) + unpack_lo<DT>(rv.x), unpack_hi<DT>(v.x) + unpack_hi<DT>(rv.x));
                            v.y = pack2<DT>(unpack_lo<DT>(v.y) + unpack_lo<DT>(rv.y), unpack_hi<DT>(v.y) + unpack_hi<DT>(rv.y));
                            v.z = pack2<DT>(unpack_lo<DT>(v.z) + unpack_lo<DT>(rv.z), unpack_hi<DT>(v.z) + unpack_hi<DT>(rv.z));
                            v.w = pack2<DT>(unpack_lo<DT>(v.w) + unpack_lo<DT>(rv.w), unpack_hi<DT>(v.w) + unpack_hi<DT>(rv.w));
                        }
                        bstore16(yrs, out_offset(bp, i) + (uint32_t)(sg * SB * 64), v);     // (out of range stays out of range)
                    }
                }
            }
        }
        __syncthreads();                                                  // t2 (in xs) and the staging area (t1s) free for the next tile
        cur = nxt;
        geo = ngeo;
    }
}

}  // namespace sbnet

using namespace sbnet;

static bool packed_is_mfma(sbnet_dtype dt, int Cin, int Cout) {
    return (dt == SBNET_BF16 || dt == SBNET_F16) && Cin % 8 == 0 && Cout % 8 == 0;
}
static size_t w32_off(int taps, int Cin, int Cout) {     // 16-byte units, same rule as sbnet_pack_weights
    const size_t CinP = ((size_t)Cin + 31) / 32 * 32, CoutP = ((size_t)Cout + 63) / 64 * 64;
    return taps * CinP * CoutP / 8;
}

template <int DT, bool FUSED, int TS, bool PRE>
static sbnet_status launch_bneck_pre(int C, const BneckParams &p, dim3 grid, hipStream_t s, const char *who) {
    switch (C) {
        case 64: hipLaunchKernelGGL((bottleneck16_kernel<DT, 64, FUSED, TS, PRE>), grid, dim3(256), 0, s, p); break;
        case 96: hipLaunchKernelGGL((bottleneck16_kernel<DT, 96, FUSED, TS, PRE>), grid, dim3(256), 0, s, p); break;
        case 128: hipLaunchKernelGGL((bottleneck16_kernel<DT, 128, FUSED, TS, PRE>), grid, dim3(256), 0, s, p); break;
        case 192: hipLaunchKernelGGL((bottleneck16_kernel<DT, 192, FUSED, TS, PRE>), grid, dim3(256), 0, s, p); break;
        case 256: hipLaunchKernelGGL((bottleneck16_kernel<DT, 256, FUSED, TS, PRE>), grid, dim3(256), 0, s, p); break;
        case 384:      // the wide form (width 65 .. 96): fused, 8 x 8 sub-tiles, no pre-activation; checked by the caller
            if constexpr (FUSED && TS == 8 && !PRE) {
                hipLaunchKernelGGL((bottleneck16_kernel<DT, 384, true, 8, false, 1, false, 384, 96>), grid, dim3(256), 0, s, p);
                break;
            }
            return fail(SBNET_EUNSUPPORTED, "%s: C = 384 only as the fused unit without pre-activation", who);
        default: return fail(SBNET_EUNSUPPORTED, "%s: C must be 64, 96, 128, 192, 256 or 384", who);
    }
    return launch_status(who);
}
template <int DT, bool FUSED, int TS>
static sbnet_status launch_bneck(int C, const BneckParams &p, dim3 grid, hipStream_t s, const char *who) {
    return p.pre_scale ? launch_bneck_pre<DT, FUSED, TS, true>(C, p, grid, s, who)
                       : launch_bneck_pre<DT, FUSED, TS, false>(C, p, grid, s, who);
}
template <int DT, bool FUSED>
static sbnet_status launch_bneck_ts(int ts, int C, const BneckParams &p, dim3 grid, hipStream_t s, const char *who) {
    return ts == 16 ? launch_bneck<DT, FUSED, 16>(C, p, grid, s, who) : launch_bneck<DT, FUSED, 8>(C, p, grid, s, who);
}

static sbnet_status bneck_entry(const char *who, bool fused, const void *in, void *out, sbnet_dtype dt, int N, int H,
                                int W, int C, int Cm, const int32_t *indices, const int32_t *count, int cap,
                                const sbnet_geom *g_in, const sbnet_geom *g_out, const void *w1, const float *b1,
                                const void *w2, const float *b2, const void *w3, const float *b3, void *stream,
                                const float *pre_scale = nullptr, const float *pre_shift = nullptr) {
    if (!in || !out || !indices || !count || !w1 || !w2 || !w3 || !b1 || !b2 || !b3)
        return fail(SBNET_EINVAL, "%s: null pointer (biases are required)", who);
    if ((pre_scale == nullptr) != (pre_shift == nullptr))
        return fail(SBNET_EINVAL, "%s: pre-activation needs both scale and shift", who);
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || Cm <= 0 || cap < 0) return fail(SBNET_EINVAL, "%s: bad sizes", who);
    if (!geom_ok(g_in) || !geom_ok(g_out)) return fail(SBNET_EINVAL, "%s: bad geometry", who);
    if (g_in->bsize_h - 2 != g_out->bsize_h || g_in->bsize_w - 2 != g_out->bsize_w)
        return fail(SBNET_EINVAL, "%s: input tile must be the output block plus a one-pixel halo", who);
    if (g_out->bstride_h < g_out->bsize_h || g_out->bstride_w < g_out->bsize_w)
        return fail(SBNET_EINVAL, "%s: output blocks must not overlap", who);
    if (fused && ranges_overlap(in, (size_t)N * H * W * C * 2, out, (size_t)N * H * W * C * 2))
        return fail(SBNET_EINVAL, "%s: y must not overlap x (use two buffers, see header)", who);
    if (((uintptr_t)in | (uintptr_t)out | (uintptr_t)w1 | (uintptr_t)w2 | (uintptr_t)w3) & 15)
        return fail(SBNET_EINVAL, "%s: pointers must be 16-byte aligned", who);
    if (dt != SBNET_BF16 && dt != SBNET_F16) return fail(SBNET_EUNSUPPORTED, "%s: dtype must be bf16 or f16", who);
    // widths up to 64 run on the kernel built for 64; C = 384 (the backbone's fourth stage, 384 / 96) on the one built for
    // 96, which needs a width above 64 (its third block of mid channels must exist in the packed weights)
    const bool wide = C == 384;
    if (Cm % 8 || (wide ? (Cm <= kCm || Cm > 96) : Cm > kCm))
        return fail(SBNET_EUNSUPPORTED, "%s: bottleneck width must be a multiple of 8, at most 64 (C = 384: 72 .. 96)", who);
    if (wide && (!fused || pre_scale)) return fail(SBNET_EUNSUPPORTED, "%s: C = 384 only as the fused unit without pre-activation", who);
    if (g_out->bsize_h % 8 || g_out->bsize_w % 8)
        return fail(SBNET_EUNSUPPORTED, "%s: block sides must be multiples of 8", who);
    if (!packed_is_mfma(dt, C, Cm)) return fail(SBNET_EUNSUPPORTED, "%s: channel counts must be multiples of 8", who);
    if (cap == 0) return SBNET_OK;
    // byte offsets inside one sample (fused) or one tile are kept in 32 bits and checked by the hardware against
    // a buffer descriptor of that size
    if ((fused ? (long long)H * W : (long long)g_in->bsize_h * g_in->bsize_w) * C >= (1LL << 30))
        return fail(SBNET_EUNSUPPORTED, "%s: a sample (or tile) must stay below 2^30 elements", who);

    BneckParams p = {};
    p.in = in; p.out = out;
    p.w1 = w1; p.w2 = w2; p.w3 = w3;
    p.w1_off = w32_off(1, C, Cm); p.w2_off = w32_off(9, Cm, Cm); p.w3_off = w32_off(1, Cm, C);
    p.b1 = b1; p.b2 = b2; p.b3 = b3;
    p.pre_scale = pre_scale; p.pre_shift = pre_shift;
    p.Cm = Cm; p.km = (Cm + 31) / 32 * 2;
    p.indices = indices; p.count = count; p.cap = cap;
    p.th = g_in->bsize_h; p.tw = g_in->bsize_w; p.oh = g_out->bsize_h; p.ow = g_out->bsize_w;
    p.H = H; p.W = W; p.Ho = H; p.Wo = W;
    p.g_in = *g_in; p.g_out = *g_out;
    // Sub-tile side: 16 x 16 where the block allows it, or 8 x 8: four times the work items at 1.56x the halo overhead
    // and a shorter latency chain each, which wins where the larger items leave most CUs idle or the last round of
    // them nearly empty.  The device decides from its count (see BneckParams); both variants are launched and one of
    // them returns at once (a few microseconds).
    const bool can16 = !wide && g_out->bsize_h % 16 == 0 && g_out->bsize_w % 16 == 0;
    const int cost8 = tuning().unit_small_item_cost_eighths;
    hipStream_t s = (hipStream_t)stream;
    for (int ts = 16; ts >= 8; ts -= 8) {
        if (ts == 16 && !can16) continue;
        p.per16 = can16 ? (p.oh / 16) * (p.ow / 16) : 0;
        p.per8 = (p.oh / 8) * (p.ow / 8);
        p.cost8 = cost8;
        p.want16 = ts == 16;
        if (can16 && ts == 16 && cost8 <= 0) continue;          // can never be chosen
        if (can16 && ts == 8 && cost8 >= 1000) continue;        // neither can this one
        p.sub_h = p.oh / ts; p.sub_w = p.ow / ts;
        p.div_sub = make_fastdiv((uint32_t)p.sub_h * p.sub_w);
        p.div_subw = make_fastdiv((uint32_t)p.sub_w);
        const long long items = (long long)cap * p.sub_h * p.sub_w;
        if (items >= (1LL << 31)) return fail(SBNET_EUNSUPPORTED, "%s: too many work items", who);
        long long gx = (items + 7) / 8 * 8;
        if (gx > 256) gx = 256;
        dim3 grid((unsigned)gx);
        sbnet_status st;
        if (dt == SBNET_BF16)
            st = fused ? launch_bneck_ts<SBNET_BF16, true>(ts, C, p, grid, s, who) : launch_bneck_ts<SBNET_BF16, false>(ts, C, p, grid, s, who);
        else
            st = fused ? launch_bneck_ts<SBNET_F16, true>(ts, C, p, grid, s, who) : launch_bneck_ts<SBNET_F16, false>(ts, C, p, grid, s, who);
        if (st != SBNET_OK) return st;
    }
    return SBNET_OK;
}

// The downsampling unit in one launch: stride 2, projected shortcut, 8 x 8 output sub-tiles.  Returns
// SBNET_EUNSUPPORTED for shapes it does not serve (the caller then composes the unit from single calls).
namespace sbnet {

template <int DT>
static sbnet_status launch_down(int C, int CO, const BneckParams &p, dim3 grid, hipStream_t s, const char *who) {
#define SBNET_DOWN(CI, CC) \
    if (C == CI && CO == CC) { hipLaunchKernelGGL((bottleneck16_kernel<DT, CI, true, 8, false, 2, true, CC>), grid, dim3(256), 0, s, p); return launch_status(who); }
    SBNET_DOWN(64, 96)
    SBNET_DOWN(96, 192)
    SBNET_DOWN(192, 256)
    SBNET_DOWN(64, 128)
    SBNET_DOWN(128, 256)
#undef SBNET_DOWN
    if (C == 256 && CO == 384) {     // width 65 .. 96 (checked by the caller)
        hipLaunchKernelGGL((bottleneck16_kernel<DT, 256, true, 8, false, 2, true, 384, 96>), grid, dim3(256), 0, s, p);
        return launch_status(who);
    }
    return fail(SBNET_EUNSUPPORTED, "%s: no one-launch downsampling unit for %d -> %d channels", who, C, CO);
}

sbnet_status unit_down_try(const char *who, const void *x, sbnet_dtype dt, int N, int H, int W, int C, int Cm, int CO,
                           const int32_t *indices, const int32_t *count, int cap, const sbnet_geom *g_in,
                           const sbnet_geom *g_out, const void *w1, const float *b1, const void *w2, const float *b2,
                           const void *w3, const float *b3, const void *ws, const float *bs, void *y, int Ho, int Wo,
                           void *stream) {
    // (the caller has checked pointers, sizes, that the geometries are those of a 3x3 with stride 2, and overlap)
    if (dt != SBNET_BF16 && dt != SBNET_F16) return fail(SBNET_EUNSUPPORTED, "%s: dtype must be bf16 or f16", who);
    const bool wide = C == 256 && CO == 384 && Cm > kCm;        // the fourth stage's 256 -> 384 / 96
    if (Cm % 8 || (wide ? Cm > 96 : Cm > kCm) || g_out->bsize_h % 8 || g_out->bsize_w % 8)
        return fail(SBNET_EUNSUPPORTED, "%s: width a multiple of 8 up to 64 (256 -> 384: 72 .. 96) and block sides multiples of 8", who);
    const bool pair = (C == 64 && CO == 96) || (C == 96 && CO == 192) || (C == 192 && CO == 256) || (C == 64 && CO == 128) ||
                      (C == 128 && CO == 256) || wide;
    if (!pair) return fail(SBNET_EUNSUPPORTED, "%s: no one-launch downsampling unit for %d -> %d channels", who, C, CO);
    if (((uintptr_t)x | (uintptr_t)y | (uintptr_t)w1 | (uintptr_t)w2 | (uintptr_t)w3 | (uintptr_t)ws) & 15)
        return fail(SBNET_EUNSUPPORTED, "%s: pointers not 16-byte aligned", who);
    if ((long long)H * W * C >= (1LL << 30) || (long long)Ho * Wo * CO >= (1LL << 30))
        return fail(SBNET_EUNSUPPORTED, "%s: a sample must stay below 2^30 elements", who);
    const long long items = (long long)cap * (g_out->bsize_h / 8) * (g_out->bsize_w / 8);
    if (items >= (1LL << 31)) return fail(SBNET_EUNSUPPORTED, "%s: too many work items", who);

    BneckParams p = {};
    p.in = x; p.out = y;
    p.w1 = w1; p.w2 = w2; p.w3 = w3; p.ws = ws;
    p.w1_off = w32_off(1, C, Cm); p.w2_off = w32_off(9, Cm, Cm); p.w3_off = w32_off(1, Cm, CO); p.ws_off = w32_off(1, C, CO);
    p.b1 = b1; p.b2 = b2; p.b3 = b3; p.bs = bs;
    p.Cm = Cm; p.km = (Cm + 31) / 32 * 2;
    p.indices = indices; p.count = count; p.cap = cap;
    p.th = g_in->bsize_h; p.tw = g_in->bsize_w; p.oh = g_out->bsize_h; p.ow = g_out->bsize_w;
    p.H = H; p.W = W; p.Ho = Ho; p.Wo = Wo;
    p.g_in = *g_in; p.g_out = *g_out;
    p.per16 = 0; p.per8 = (p.oh / 8) * (p.ow / 8); p.cost8 = 8; p.want16 = 0;
    p.sub_h = p.oh / 8; p.sub_w = p.ow / 8;
    p.div_sub = make_fastdiv((uint32_t)p.sub_h * p.sub_w);
    p.div_subw = make_fastdiv((uint32_t)p.sub_w);
    long long gx = (items + 7) / 8 * 8;
    if (gx > 256) gx = 256;
    dim3 grid((unsigned)gx);
    return dt == SBNET_BF16 ? launch_down<SBNET_BF16>(C, CO, p, grid, (hipStream_t)stream, who)
                            : launch_down<SBNET_F16>(C, CO, p, grid, (hipStream_t)stream, who);
}

}  // namespace sbnet

extern "C" sbnet_status sbnet_bottleneck_on_tiles(const void *tiles_in, sbnet_dtype dtype, int H, int W, int C, int Cm,
                                                  const int32_t *indices, const int32_t *count, int cap,
                                                  const sbnet_geom *g_in, const sbnet_geom *g_out, const void *w1,
                                                  const float *b1, const void *w2, const float *b2, const void *w3,
                                                  const float *b3, void *tiles_out, void *stream) {
    return bneck_entry("sbnet_bottleneck_on_tiles", false, tiles_in, tiles_out, dtype, 1, H, W, C, Cm, indices, count,
                       cap, g_in, g_out, w1, b1, w2, b2, w3, b3, stream);
}

extern "C" sbnet_status sbnet_sparse_bottleneck(const void *x, sbnet_dtype dtype, int N, int H, int W, int C, int Cm,
                                                const int32_t *indices, const int32_t *count, int cap,
                                                const sbnet_geom *g_in, const sbnet_geom *g_out, const void *w1,
                                                const float *b1, const void *w2, const float *b2, const void *w3,
                                                const float *b3, void *y, void *stream) {
    return bneck_entry("sbnet_sparse_bottleneck", true, x, y, dtype, N, H, W, C, Cm, indices, count, cap, g_in, g_out,
                       w1, b1, w2, b2, w3, b3, stream);
}

extern "C" sbnet_status sbnet_bottleneck_on_tiles_preact(const void *tiles_in, sbnet_dtype dtype, int H, int W, int C,
                                                         int Cm, const int32_t *indices, const int32_t *count, int cap,
                                                         const sbnet_geom *g_in, const sbnet_geom *g_out,
                                                         const float *pre_scale, const float *pre_shift, const void *w1,
                                                         const float *b1, const void *w2, const float *b2,
                                                         const void *w3, const float *b3, void *tiles_out, void *stream) {
    if (!pre_scale || !pre_shift) return fail(SBNET_EINVAL, "sbnet_bottleneck_on_tiles_preact: null pointer");
    return bneck_entry("sbnet_bottleneck_on_tiles_preact", false, tiles_in, tiles_out, dtype, 1, H, W, C, Cm, indices,
                       count, cap, g_in, g_out, w1, b1, w2, b2, w3, b3, stream, pre_scale, pre_shift);
}

extern "C" sbnet_status sbnet_sparse_bottleneck_preact(const void *x, sbnet_dtype dtype, int N, int H, int W, int C, int Cm,
                                                       const int32_t *indices, const int32_t *count, int cap,
                                                       const sbnet_geom *g_in, const sbnet_geom *g_out,
                                                       const float *pre_scale, const float *pre_shift, const void *w1,
                                                       const float *b1, const void *w2, const float *b2, const void *w3,
                                                       const float *b3, void *y, void *stream) {
    if (!pre_scale || !pre_shift) return fail(SBNET_EINVAL, "sbnet_sparse_bottleneck_preact: null pointer");
    return bneck_entry("sbnet_sparse_bottleneck_preact", true, x, y, dtype, N, H, W, C, Cm, indices, count, cap, g_in,
                       g_out, w1, b1, w2, b2, w3, b3, stream, pre_scale, pre_shift);
}
