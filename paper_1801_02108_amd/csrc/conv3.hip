// 3x3 tile convolution for any stride and tile size, bf16 / f16 with channel counts that are multiples of 8, and
// the pointwise (1x1) convolution with input channels in multiples of 64 through the same pipeline
// (Sec. 3.2 of arXiv 1801.02108: the regular convolution that runs on every gathered block, here also for the
// stride-2 geometry of Fig. 3 and the wider layers of the later backbone stages; in fused mode also the gather
// before it and the scatter / scatter-add after it, Sec. 3.4).
//
// Design for gfx950: an implicit GEMM tiled through LDS, both operands read from LDS.
//   * Measured on MI355X: with one wave per SIMD a stream of 32x32x16 MFMAs that takes BOTH operands from LDS
//     (two 16-byte-per-lane reads per MFMA, conflict-free) still runs at 94 % of the rate of a register-only
//     stream.  So nothing has to stay in registers across MFMAs and the matrix loop never waits on memory: a
//     chunk of CC input channels of the input rows AND of the weights of the workgroup's 64 output channels sits
//     in LDS, and the loop only reads LDS.
//   * A work item is (active block, pass of PP output pixels, group of 64 output channels); a workgroup walks its
//     items and, inside an item, the chunks of CC input channels.  Chunks are double-buffered in LDS and pipelined
//     two deep through registers: while the matrix cores work on chunk i, a thread writes its vectors of chunk i+1
//     (loaded during chunk i-1) to the other LDS buffer and, into the registers this frees, requests the same
//     vectors of chunk i+2 (of a following item past the last chunk).
//   * 3x3: eight waves, two per SIMD, with separate roles: four run the matrix steps and store the results, four
//     do the staging.  (A wave stands at the issue of a load while the CU's address unit is busy; with one wave
//     per SIMD doing both, one or two staging vectors per MFMA step, a chunk took the sum of its matrix, LDS and
//     load time.)  1x1: four waves that do both and two workgroups per CU.
//   * All global traffic goes through buffer descriptors: halo pixels outside the image, vectors past the end of
//     the staged rows and channels past Cin read as zeros, stores outside the image or past Cout are dropped.  No
//     branch surrounds a load, so the compiler's wait counts stay exact.
//   * Columns are staged de-interleaved by stride phase (column x goes to plane x % sw, slot x / sw), which turns
//     the stride-sw walk of a fragment read into consecutive LDS pixels: the same conflict-free pattern for every
//     stride.  The LDS pixel stride is the chunk's channels + 16 B pad.
//   * Results are transposed through a wave-private LDS area, 32 pixels x 32 channels at a time, so that a store
//     instruction writes 64-byte runs instead of 16-byte pieces.
//   * Workgroup tiles: 256 pixels x 64 channels (wave: 64 px x 64 ch, 4 accumulators), 128 x 64 for problems
//     where that means fewer rounds of work on the device (picked on the device from the active count: one launch
//     holds both shapes), 384 x 64 beside 256 x 64 for blocks of 257 ... 384 output pixels (the 18x18 outputs of a
//     data gradient on 16x16 blocks), 64 x 64 for tiles of at most 64 output pixels, and for strided tiles 128 pixels x
//     96 / 128 channels where the channel count is a multiple of that (beside 128 x 64 in the same launch).  Chunks of 32 channels where two
//     buffers of that fit in LDS (stride 1), else of 16 (the 33x33 input tile of a strided 16x16 block).
#include "conv_common.h"

#include <type_traits>

namespace sbnet {

constexpr int kLds3 = 160 * 1024;
constexpr int kDump3 = 4096;                 // one 16-byte slot per thread for staging vectors that have no place
constexpr int kOst3Ps = 80;                  // result transpose: bytes per pixel (32 channels + 16 B pad)
constexpr int kOst3 = 32 * kOst3Ps;          // ... per wave

struct Plan3 {
    int mpasses, ngroups;
    FastDiv div_pt, div_ng, div_sw, div_nch;
    int cpp;                 // LDS pixel slots per column phase: ceil(tw / sw)
    uint32_t nvec_in;        // 16-byte vectors of one input chunk
    int nchunks;
    uint32_t buf_bytes;      // one LDS buffer: input chunk, then weight chunk
    uint32_t w_off;          // offset of the weight chunk inside a buffer
    uint32_t dump_off, ost_off, bias_off;    // after the two buffers
    uint32_t w_bytes;        // bytes of the 32x32x16 operand copy of the weights
    int ks16;                // 16-channel k-steps per output group: 9 * CinP / 16
};

struct Item3 {
    uint32_t b;
    int pass, ng;
    int n, by, bx;
};

struct Src3 {
    const void *base;        // the sample (fused) or tile the rows come from
    uint32_t origin;         // byte offset of staged pixel (0, 0); wraps below zero above / left of the image
    int gx0;                 // image column of staged column 0
    int ng;
};

struct Chunk3 {
    const void *base;
    uint32_t origin;         // ... of channel c0
    int gx0;
    int c0;
    uint32_t wofs;           // byte offset of (group, tap 0, channel c0) in the packed weights (wide groups: of channel c0 only)
    int nb0;                 // first 32-channel block of the group
};

// KH = 3: the 3x3 kernel this file is named for; KH = 1: pointwise convolutions through the same pipeline (one tap,
// chunks of 64 channels so that a chunk still holds several MFMA steps; of 32 for channel counts that need it).
//
// SPEC: the workgroup has eight waves, two per SIMD, with separate roles.  Waves 0-3 only read fragments from LDS,
// run the matrix steps and store the results; waves 4-7 only move chunks (memory -> registers -> LDS).  A wave is
// held at the issue of a load while the CU's address unit is busy and at the wait in front of an LDS write, and with
// one wave per SIMD the matrix core stood idle through both: per chunk the kernel took about the SUM of its matrix,
// LDS and load time.  With the roles in different waves of the same SIMD they overlap.  Both roles walk the same
// chunk sequence and meet at the same barrier per chunk.
template <int DT, bool FUSED, bool ADD, int CC, int WP, int CBW, int PBW, int NVI, int KH = 3, bool SPEC = false>
__device__ __forceinline__ void conv3_body(const ConvParams &p, const Plan3 &q) {
    static_assert(FUSED || !ADD, "adding into the output is part of the fused form");
    // Register sets for chunks in flight.  Two (requests two chunks further ahead) were measured for the small
    // workgroup tiles and gained nothing: the compiler's wait before a vector's LDS write allows only one set's
    // worth of younger loads, and those tiles are bound by the issue of their staging instructions anyway.
    constexpr int RS = 1;
    constexpr int CV = CC / 8;                       // 16-byte vectors per pixel and chunk
    constexpr int KST = CC / 16;                     // k-steps of 16 channels per tap
    constexpr int TAPS = KH * KH;
    constexpr int NS = TAPS * KST;                   // MFMA steps per chunk
    constexpr int PS = CC * 2 + 16;                  // LDS bytes per input pixel
    constexpr int NB = (4 / WP) * CBW;               // blocks of 32 output channels per group: 2, or 3 / 4 (wide groups)
    constexpr int GW = NB * 32;                      // output channels per group
    constexpr int WVEC = NS * NB * 64;               // vectors of a weight chunk: steps x NB blocks of 32 channels x 64 lanes
    constexpr int NVW = (WVEC + 255) / 256;
    constexpr int NV = NVI + NVW;                    // staging vectors per thread and chunk
    constexpr int PER = (NV + NS - 1) / NS;          // ... handled per MFMA step
    constexpr int PP = WP * PBW * 32;                // output pixels per pass
    constexpr int NM = CBW * PBW;                    // MFMAs per step
    constexpr int D0 = NM >= 4 ? 2 : (NM == 3 ? 3 : (NM == 2 ? 4 : 8));
    constexpr int D = D0 < NS ? D0 : NS - 1;         // steps the fragment reads run ahead of the MFMAs
    extern __shared__ __align__(16) unsigned char lds[];

    constexpr int NT = SPEC ? 512 : 256;             // threads of the workgroup
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool mover = !SPEC || wave_all >= 4;       // stages chunks
    const int wave = wave_all & 3;                   // number among the waves of its role
    const int stid = tid & 255;                      // ... thread among the 256 that stage
    const int g = lane >> 5, m = lane & 31;          // k-group / channel half, pixel within a fragment
    const int pw = wave % WP, cw = wave / WP;
    const int M = p.oh * p.ow;

    const int nact = max(min(*p.count, p.cap), 0);
    const uint32_t per_tile = (uint32_t)q.mpasses * q.ngroups;
    const uint32_t items = (uint32_t)nact * per_tile;
    const uint32_t G = gridDim.x;                    // multiple of 8
    // workgroups are dealt round-robin to the 8 XCDs: give each XCD a contiguous run of items (the passes and
    // channel groups of one block, and neighbouring blocks, share input lines in that XCD's L2)
    const uint32_t first = (blockIdx.x & 7) * (G >> 3) + (blockIdx.x >> 3);
    if (first >= items) return;
    const uint32_t last = items - 1u;

    // A work item's index triple is requested three items ahead.  The address is the same in every lane, but the
    // loads are issued as per-lane loads and left in vector registers (the opaque zero hides the uniformity): a
    // value the compiler knows to be uniform is moved to a scalar register right after the load, which stalls
    // the wave for a memory round trip on the spot.  It is made scalar (resolve) behind a point where younger
    // loads have been waited for anyway.
    int lane_zero = 0;
    asm volatile("" : "+v"(lane_zero));
    auto request = [&](uint32_t it) __attribute__((always_inline)) {
        Item3 c;
        c.b = fdiv(it, q.div_pt);
        const uint32_t rest = it - c.b * per_tile;
        c.pass = (int)fdiv(rest, q.div_ng);
        c.ng = (int)rest - c.pass * q.ngroups;
        c.n = c.by = c.bx = 0;
        if (FUSED) {
            const int32_t *t = p.indices + 3 * (size_t)c.b + lane_zero;
            c.n = t[0];
            c.by = t[1];
            c.bx = t[2];
        }
        return c;
    };
    auto resolve = [&](const Item3 &c) __attribute__((always_inline)) {
        Item3 r = c;
        if (FUSED) {
            r.n = __builtin_amdgcn_readfirstlane(c.n);
            r.by = __builtin_amdgcn_readfirstlane(c.by);
            r.bx = __builtin_amdgcn_readfirstlane(c.bx);
        }
        return r;
    };
    const int in_w = FUSED ? p.W : p.tw;                          // pixels per row of the addressed array
    const uint32_t in_bytes = (uint32_t)(FUSED ? p.H : p.th) * in_w * p.Cin * 2u;   // one sample / one tile
    auto source = [&](const Item3 &c) __attribute__((always_inline)) {
        Src3 s;
        const int r_lo = (int)fdiv((uint32_t)c.pass * PP, p.div_ow) * p.sh;          // first input row of the pass
        const uint16_t *base = (const uint16_t *)p.in;
        if (FUSED) {
            const int y0 = p.g_in.boffset_h + c.by * p.g_in.bstride_h + r_lo;
            const int x0 = p.g_in.boffset_w + c.bx * p.g_in.bstride_w;
            base += (long long)c.n * p.H * p.W * p.Cin;
            s.origin = (uint32_t)((y0 * in_w + x0) * p.Cin) * 2u;
            s.gx0 = x0;
        } else {
            base += (long long)c.b * p.th * p.tw * p.Cin;
            s.origin = (uint32_t)(r_lo * in_w * p.Cin) * 2u;
            s.gx0 = 0;
        }
        s.base = base;
        s.ng = c.ng;
        return s;
    };

    // ---- staging plan, the same for every chunk.  Input vector u of this thread is 16 bytes (8 channels) of pixel
    //      (tid + 256 u) / CV of the staged rows, row-major; a vector past the end gets a column no image has
    //      (so it loads zeros) and the dump slot.  Weight vector u is vector tid + 256 u of the chunk's fragments.
    //      LDS address of a vector = lbase + (buffer number) * lstep.
    uint32_t gdelta[NVI], lbase[NV], lstep[NV], wsrc[NVW];
    int colv[NVI];
    const int c8 = stid % CV;
    const int cin16 = p.CinP >> 4;
#pragma unroll
    for (int u = 0; u < NVI; ++u) {
        const uint32_t v = (uint32_t)stid + 256u * u;
        const uint32_t px = v / CV;
        const uint32_t row = fdiv(px, p.div_tw), col = px - row * p.tw;
        const uint32_t cq = fdiv(col, q.div_sw), cr = col - cq * p.sw;
        const bool ok = v < q.nvec_in;
        lbase[u] = ok ? ((row * p.sw + cr) * q.cpp + cq) * PS + c8 * 16 : q.dump_off + stid * 16;
        lstep[u] = ok ? q.buf_bytes : 0u;
        gdelta[u] = (uint32_t)((row * in_w + col) * p.Cin + c8 * 8) * 2u;
        colv[u] = ok ? (int)col : 0x40000000;
    }
    // The packed weights are [group of 64 channels][tap][16-channel step][32-channel half][lane] x 16 bytes; a chunk in
    // LDS is [step][block of the group][lane].  With 64-channel groups a tap's steps of a chunk are one contiguous run.
    // Wide groups (96 / 128 channels) take their blocks from two 64-channel groups: block b of group ng is half
    // (ng NB + b) & 1 of 64-group (ng NB + b) >> 1, worked out per vector when it is requested (wblk: b, or -1 for none).
    int wblk[NVW];
#pragma unroll
    for (int u = 0; u < NVW; ++u) {
        const uint32_t v = (uint32_t)stid + 256u * u;
        const bool ok = v < (uint32_t)WVEC;
        lbase[NVI + u] = ok ? q.w_off + v * 16 : q.dump_off + stid * 16;
        lstep[NVI + u] = ok ? q.buf_bytes : 0u;
        if (NB == 2) {
            const uint32_t tap = v / (KST * 128), rem = v % (KST * 128);
            wsrc[u] = ok ? (tap * cin16 * 128u + rem) * 16u : kOutOfRange;
            wblk[u] = 0;
        } else {
            const uint32_t st = v / (NB * 64), b = (v / 64) % NB, ln = v % 64;
            const uint32_t tap = st / KST, k = st % KST;
            wsrc[u] = (tap * cin16 + k) * 2048u + ln * 16u;
            wblk[u] = ok ? (int)b : -1;
        }
    }
    const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc(
        (void *)((const uint4 *)p.w + p.w32_offset), 0, (int)q.w_bytes, (int)kBufWord3);

    uint4 stage[RS][NV];
    // Rows outside the image fall outside the descriptor by themselves; columns outside would wrap into the
    // neighbouring row and channels past Cin into the neighbouring pixel, so those get the out-of-range offset.
    auto issue1 = [&](int r, int u, const Chunk3 &ch, bool chan_ok) __attribute__((always_inline)) {
        if (u < NVI) {
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)ch.base, 0, (int)in_bytes, (int)kBufWord3);
            const bool ok = chan_ok && (uint32_t)(ch.gx0 + colv[u]) < (uint32_t)in_w;
            stage[r][u] = buf_load16(rs, ok ? ch.origin + gdelta[u] : kOutOfRange);
        } else if (NB == 2) {
            stage[r][u] = buf_load16(wrs, wsrc[u - NVI] + ch.wofs);
        } else {
            const uint32_t nbk = (uint32_t)(ch.nb0 + wblk[u - NVI]);
            const uint32_t off = (nbk >> 1) * (uint32_t)q.ks16 * 2048u + (nbk & 1u) * 1024u + wsrc[u - NVI] + ch.wofs;
            stage[r][u] = buf_load16(wrs, wblk[u - NVI] >= 0 ? off : kOutOfRange);
        }
    };
    auto write1 = [&](int r, int u, uint32_t bufno) __attribute__((always_inline)) {
        *(uint4 *)(lds + lbase[u] + bufno * lstep[u]) = stage[r][u];
    };
    auto chunk_of = [&](const Src3 &s, int c) __attribute__((always_inline)) {
        Chunk3 ch;
        ch.base = s.base;
        ch.c0 = c * CC;
        ch.origin = s.origin + (uint32_t)ch.c0 * 2u;
        ch.gx0 = s.gx0;
        ch.wofs = NB == 2 ? (uint32_t)(s.ng * q.ks16 + (ch.c0 >> 4)) * 2048u : (uint32_t)(ch.c0 >> 4) * 2048u;
        ch.nb0 = s.ng * NB;
        return ch;
    };

    // ---- the workgroup's chunks, numbered gi = 0, 1, ... over its items: chunk gi is chunk gi % nchunks of item
    //      first + (gi / nchunks) * G (past the end: the last item again, staged but never used).  RS + 2 are
    //      known at any time: line[0] is the one the matrix cores work on, line[1] is on its way from registers to
    //      LDS, line[RS + 1] is being requested; the index triple of one more is in flight.
    struct Work3 {
        Item3 it;
        Src3 s;
        int c;
    };
    auto request_chunk = [&](uint32_t gi) __attribute__((always_inline)) {
        Work3 w;
        const uint32_t k = fdiv(gi, q.div_nch);
        w.c = (int)(gi - k * q.nchunks);
        w.it = request(min(first + k * G, last));
        return w;
    };
    auto resolve_chunk = [&](const Work3 &r) __attribute__((always_inline)) {
        Work3 w;
        w.c = r.c;
        w.it = resolve(r.it);
        w.s = source(w.it);
        return w;
    };
    Work3 line[RS + 2];
#pragma unroll
    for (int k = 0; k < RS + 2; ++k) line[k] = request_chunk(k);
#pragma unroll
    for (int k = 0; k < RS + 2; ++k) line[k] = resolve_chunk(line[k]);
    const uint32_t nwork = ((last - first) / G + 1u) * (uint32_t)q.nchunks;     // chunks of this workgroup

    // chunk k lives in register set k % RS: chunks 0 .. RS-1 are requested at once, chunk 0 goes to LDS buffer 0 and
    // chunk RS takes its registers
    if (mover) {
#pragma unroll
        for (int r = 0; r < RS; ++r) {
            const Chunk3 ch = chunk_of(line[r].s, line[r].c);
            const bool chan_ok = ch.c0 + c8 * 8 < p.Cin;
#pragma unroll
            for (int u = 0; u < NV; ++u) issue1(r, u, ch, chan_ok);
        }
    }
    // bias of all groups -> LDS (zeros past Cout or without bias)
    {
        float *bl = (float *)(lds + q.bias_off);
        for (int i = tid; i < q.ngroups * GW; i += NT) bl[i] = (p.bias && i < p.Cout) ? p.bias[i] : 0.f;
    }
    // tap offsets in the de-interleaved layout
    uint32_t tapoff[TAPS];
#pragma unroll
    for (int r = 0; r < KH; ++r)
#pragma unroll
        for (int t = 0; t < KH; ++t) tapoff[r * KH + t] = (uint32_t)((r * p.sw + t % p.sw) * q.cpp + t / p.sw) * PS;
    uint32_t floor16 = p.relu ? 0u : 0x80008000u;    // ReLU on a pair of rounded values: integer max with 0 (or with -32768: identity)
    asm volatile("" : "+s"(floor16));
    int floor_i = p.relu ? 0 : (int)0x80000000;
    asm volatile("" : "+s"(floor_i));
    if (mover) {
#pragma unroll
        for (int u = 0; u < NV; ++u) write1(0, u, 0);
        const Chunk3 ch = chunk_of(line[RS].s, line[RS].c);
        const bool chan_ok = ch.c0 + c8 * 8 < p.Cin;
#pragma unroll
        for (int u = 0; u < NV; ++u) issue1(0, u, ch, chan_ok);
    }
    __syncthreads();

    uint32_t par = 0;                                // LDS buffer the matrix work reads
    unsigned char *ost = lds + q.ost_off + wave * kOst3;
    f32x16 acc[CBW][PBW];
    uint32_t p_lo = 0;
    uint32_t xbase[PBW];
    // one chunk: register set R = (gi + 1) % RS holds chunk gi + 1 on entry and chunk gi + RS + 1 on exit.
    // ROLE 0: matrix steps with the staging between them; 1: matrix steps and results only; 2: staging only.
    auto chunk_body = [&](auto r_tag, auto role_tag, uint32_t gi) __attribute__((always_inline)) {
        constexpr int R = decltype(r_tag)::value;
        constexpr int ROLE = decltype(role_tag)::value;
        constexpr bool MM = ROLE != 2, ST = ROLE != 1;
        const Work3 rq = request_chunk(gi + RS + 2);
        const Work3 cur = line[0];
        const bool firstc = cur.c == 0, lastc = cur.c + 1 == q.nchunks;
        {
            const Chunk3 aheadc = chunk_of(line[RS + 1].s, line[RS + 1].c);
            const bool chan_ok = aheadc.c0 + c8 * 8 < p.Cin;
            const unsigned char *B = lds + par * q.buf_bytes;
            if (!MM) {
#pragma unroll
                for (int u = 0; u < NV; ++u) {
                    write1(R, u, par ^ 1u);
                    issue1(R, u, aheadc, chan_ok);
                }
            }
            if (MM && firstc) {
                // this lane's pixels: block pb of the wave is 32 consecutive output pixels of the pass
                p_lo = (uint32_t)cur.it.pass * PP;
                const uint32_t i_lo = fdiv(p_lo, p.div_ow);
#pragma unroll
                for (int pb = 0; pb < PBW; ++pb) {
                    const uint32_t px = min(p_lo + (uint32_t)((pw * PBW + pb) * 32 + m), (uint32_t)M - 1u);
                    const uint32_t i = fdiv(px, p.div_ow), j = px - i * p.ow;
                    xbase[pb] = ((i - i_lo) * p.sh * p.sw * q.cpp + j) * PS + g * 16;
                }
                // accumulators start from the bias
#pragma unroll
                for (int cb = 0; cb < CBW; ++cb) {
                    const float4 *bl = (const float4 *)(lds + q.bias_off) + (cur.it.ng * GW + (cw * CBW + cb) * 32 + g * 16) / 4;
#pragma unroll
                    for (int k4 = 0; k4 < 4; ++k4) {
                        const float4 bv = bl[k4];
#pragma unroll
                        for (int pb = 0; pb < PBW; ++pb) {
                            acc[cb][pb][k4 * 4 + 0] = bv.x; acc[cb][pb][k4 * 4 + 1] = bv.y;
                            acc[cb][pb][k4 * 4 + 2] = bv.z; acc[cb][pb][k4 * 4 + 3] = bv.w;
                        }
                    }
                }
            }

            // ---- matrix work of the chunk: step s = (tap, 16-channel step); A = weights (32 channels x 16 k),
            //      B = 32 pixels x 16 k; fragment reads run D steps ahead.  Between the MFMAs of a step: PER
            //      staging vectors of the next chunk go to the other buffer and are requested again for the
            //      chunk after it.
            if (MM) {
                const unsigned char *WL = B + q.w_off + (cw * CBW) * 1024 + lane * 16;
                uint4 xa[D + 1][CBW], xb[D + 1][PBW];
                auto read = [&](int s) __attribute__((always_inline)) {
                    const int slot = s % (D + 1);
#pragma unroll
                    for (int cb = 0; cb < CBW; ++cb) xa[slot][cb] = *(const uint4 *)(WL + (s * NB + cb) * 1024);
#pragma unroll
                    for (int pb = 0; pb < PBW; ++pb)
                        xb[slot][pb] = *(const uint4 *)(B + xbase[pb] + tapoff[s / KST] + (s % KST) * 32);
                };
#pragma unroll
                for (int s = 0; s < D; ++s) read(s);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    if (s + D < NS) read(s + D);
#pragma unroll
                    for (int cb = 0; cb < CBW; ++cb)
#pragma unroll
                        for (int pb = 0; pb < PBW; ++pb) {
                            acc[cb][pb] = mfma32x32x16<DT>(xa[s % (D + 1)][cb], xb[s % (D + 1)][pb], acc[cb][pb]);
                            if (ST && cb * PBW + pb < PER) {
                                const int u = s * PER + cb * PBW + pb;
                                if (u < NV) {
                                    write1(R, u, par ^ 1u);
                                    issue1(R, u, aheadc, chan_ok);
                                }
                            }
                        }
                    if (ST && PER > NM) {
#pragma unroll
                        for (int e = NM; e < PER; ++e) {
                            const int u = s * PER + e;
                            if (u < NV) {
                                write1(R, u, par ^ 1u);
                                issue1(R, u, aheadc, chan_ok);
                            }
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }

            // ---- epilogue after the last chunk: ReLU, optional add, NHWC stores.  A lane holds 16 consecutive
            //      channels of one pixel per accumulator; 32 pixels x 32 channels at a time go through the wave's
            //      LDS area and come back as 64 contiguous bytes per four lanes.  Pixels past the end of the tile,
            //      columns outside the image and channels past Cout get the out-of-range offset; rows outside fall
            //      outside the descriptor.
            if (MM && lastc) {
                uint16_t *obase = (uint16_t *)p.out;
                uint32_t obytes, origin;
                int ox0 = 0, out_w;
                if (FUSED) {
                    const int oy0 = p.g_out.boffset_h + cur.it.by * p.g_out.bstride_h;
                    ox0 = p.g_out.boffset_w + cur.it.bx * p.g_out.bstride_w;
                    out_w = p.Wo;
                    obase += (long long)cur.it.n * p.Ho * p.Wo * p.Cout;
                    obytes = (uint32_t)p.Ho * p.Wo * p.Cout * 2u;
                    origin = (uint32_t)((oy0 * p.Wo + ox0) * p.Cout) * 2u;
                } else {
                    out_w = p.ow;
                    obase += (long long)cur.it.b * M * p.Cout;
                    obytes = (uint32_t)M * p.Cout * 2u;
                    origin = 0;
                }
                const __amdgpu_buffer_rsrc_t ors = __builtin_amdgcn_make_buffer_rsrc((void *)obase, 0, (int)obytes, (int)kBufWord3);
                auto pixel_offset = [&](uint32_t px, bool &ok) __attribute__((always_inline)) {
                    const uint32_t pc = min(px, (uint32_t)M - 1u);
                    const uint32_t i = fdiv(pc, p.div_ow), j = pc - i * p.ow;
                    ok = px < (uint32_t)M && (!FUSED || (uint32_t)(ox0 + (int)j) < (uint32_t)p.Wo);
                    return origin + (uint32_t)((i * out_w + j) * p.Cout) * 2u;
                };
                const int chg = cur.it.ng * GW + cw * CBW * 32;                    // first channel of the wave
#pragma unroll
                for (int pb = 0; pb < PBW; ++pb) {
                    const uint32_t pblock = p_lo + (uint32_t)((pw * PBW + pb) * 32);
                    uint4 old[CBW][2];
                    if (ADD) {      // read in the MFMA layout, so that the sum is formed in fp32 and rounded once
                        bool ok1;
                        const uint32_t off1 = pixel_offset(pblock + m, ok1);
#pragma unroll
                        for (int cb = 0; cb < CBW; ++cb)
#pragma unroll
                            for (int h = 0; h < 2; ++h) {
                                const int ch = chg + cb * 32 + g * 16 + h * 8;
                                old[cb][h] = buf_load16(ors, (ok1 && ch < p.Cout) ? off1 + (uint32_t)ch * 2u : kOutOfRange);
                            }
                    }
                    bool ok2[2];
                    uint32_t off2[2];
#pragma unroll
                    for (int j = 0; j < 2; ++j) off2[j] = pixel_offset(pblock + j * 16 + (lane >> 2), ok2[j]);
#pragma unroll
                    for (int cb = 0; cb < CBW; ++cb) {
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            uint32_t w[4];
                            if (ADD) {
                                float v[8];
#pragma unroll
                                for (int k = 0; k < 8; ++k) v[k] = __int_as_float(max(__float_as_int(acc[cb][pb][h * 8 + k]), floor_i));
                                const uint4 o = old[cb][h];
                                v[0] += unpack_lo<DT>(o.x); v[1] += unpack_hi<DT>(o.x);
                                v[2] += unpack_lo<DT>(o.y); v[3] += unpack_hi<DT>(o.y);
                                v[4] += unpack_lo<DT>(o.z); v[5] += unpack_hi<DT>(o.z);
                                v[6] += unpack_lo<DT>(o.w); v[7] += unpack_hi<DT>(o.w);
#pragma unroll
                                for (int k = 0; k < 4; ++k) w[k] = pack2<DT>(v[2 * k], v[2 * k + 1]);
                            } else {
#pragma unroll
                                for (int k = 0; k < 4; ++k)
                                    w[k] = relu_pair(pack2<DT>(acc[cb][pb][h * 8 + 2 * k], acc[cb][pb][h * 8 + 2 * k + 1]), floor16);
                            }
                            *(uint4 *)(ost + m * kOst3Ps + g * 32 + h * 16) = make_uint4(w[0], w[1], w[2], w[3]);
                        }
                        __builtin_amdgcn_wave_barrier();     // LDS serves one wave's accesses in order: no wait needed
                        const int ch = chg + cb * 32 + (lane & 3) * 8;
#pragma unroll
                        for (int j = 0; j < 2; ++j) {
                            const uint4 v = *(const uint4 *)(ost + (j * 16 + (lane >> 2)) * kOst3Ps + (lane & 3) * 16);
                            buf_store16(ors, (ok2[j] && ch < p.Cout) ? off2[j] + (uint32_t)ch * 2u : kOutOfRange, v);
                        }
                        __builtin_amdgcn_wave_barrier();
                    }
                }
            }
        }
        const Work3 nxt = resolve_chunk(rq);             // the loads waited for in this chunk are younger than its request
        __syncthreads();
        par ^= 1u;
#pragma unroll
        for (int k = 0; k < RS + 1; ++k) line[k] = line[k + 1];
        line[RS + 1] = nxt;
    };
    static_assert(RS == 1, "the loops below step one chunk at a time");
    using Set0 = std::integral_constant<int, 0>;
    if (!SPEC) {
        for (uint32_t gi = 0; gi < nwork; ++gi) chunk_body(Set0{}, std::integral_constant<int, 0>{}, gi);
    } else if (wave_all < 4) {
        for (uint32_t gi = 0; gi < nwork; ++gi) chunk_body(Set0{}, std::integral_constant<int, 1>{}, gi);
    } else {
        for (uint32_t gi = 0; gi < nwork; ++gi) chunk_body(Set0{}, std::integral_constant<int, 2>{}, gi);
    }
}

template <int DT, bool FUSED, bool ADD, int CC, int WP, int CBW, int PBW, int NVI>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void conv3_kernel(ConvParams p, Plan3 q) {
    conv3_body<DT, FUSED, ADD, CC, WP, CBW, PBW, NVI, 3, true>(p, q);
}

// Pointwise convolutions wait on memory, not on the matrix cores: their kernel is built for two workgroups per CU
// (at most 256 registers, and the host picks a tile shape whose LDS plan fits twice).
template <int DT, bool FUSED, bool ADD, int CC, int WP, int CBW, int PBW, int NVI>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void conv3_pointwise_kernel(ConvParams p, Plan3 q) {
    conv3_body<DT, FUSED, ADD, CC, WP, CBW, PBW, NVI, 1, false>(p, q);
}

// The 256-pixel and the 128-pixel tile shape in one launch: the device-side count picks one (rounds of work on 256
// CUs with either shape; an item of the smaller tile costs about 5/8 of a larger one: half the matrix work, the same
// weights to stage; the ratio comes with the launch, in eighths).  Two separate launches, of which one returns, cost a launch more.
// PBWB = 3, PBWS = 2: the shapes are 384 and 256 pixels (three / two pixel blocks per wave), for tiles of 257 ... 384
// output pixels such as the 18x18 of a data gradient on 16x16 blocks: one item per tile instead of three of 128 pixels,
// each of which staged the tile's rows and the weights again; two items of 256 pixels where those fill the device in
// one round.
// CBWP = 3 / 4: groups of 96 / 128 output channels (three / four channel blocks per wave): the input rows of an item are
// staged once for 96 / 128 channels instead of once per 64, a 96-channel layer does not pay for a half-empty second
// group, and a wave reads 5 / 6 fragments per 6 / 8 MFMAs instead of 4 per 4.  Their weight chunks are larger, so
// these run on 16-channel chunks.
template <int DT, bool FUSED, bool ADD, int CCB, int NVIB, int CCS, int NVIS, int PBWB = 2, int PBWS = 1, int CBWP = 2>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void conv3_pair_kernel(ConvParams p, Plan3 qb, Plan3 qs) {
    const int nact = max(min(*p.count, p.cap), 0);
    const uint32_t per_big = (uint32_t)qb.mpasses * qb.ngroups, per_small = (uint32_t)qs.mpasses * qs.ngroups;
    const uint32_t rb = ((uint32_t)nact * per_big + 255u) >> 8, rs = ((uint32_t)nact * per_small + 255u) >> 8;
    // the ratio is given for the 128- against the 256-pixel item (5/8 as measured); a 256-pixel item against a
    // 384-pixel one is taken as 6/8 (on the 18x18 outputs of a data gradient one round of either took 12.2 and 14.9 us)
    const uint32_t cost8 = PBWB == 3 ? ((uint32_t)p.small_cost8 * 6u + 2u) / 5u : (uint32_t)p.small_cost8;
    if ((unsigned long long)rb * 8u <= (unsigned long long)rs * cost8) conv3_body<DT, FUSED, ADD, CCB, 4, CBWP, PBWB, NVIB, 3, true>(p, qb);
    // (128 pixels x 128 channels: a wave takes 64 x 64, four fragment reads per four MFMAs, rather than 32 x 128, five)
    else if (CBWP == 4 && PBWS == 1) conv3_body<DT, FUSED, ADD, CCS, 2, 2, 2, NVIS, 3, true>(p, qs);
    else conv3_body<DT, FUSED, ADD, CCS, 4, CBWP, PBWS, NVIS, 3, true>(p, qs);
}

// 128-pixel items with groups of 96 / 128 output channels or of 64 in one launch, for strided tiles whose 256-pixel shape
// has no room for the wider weight chunks (the 33x33 input tile of a 16x16 block).  Measured (192 -> 256 channels, stride
// 2): with up to ~25 active blocks the 64-channel items are faster (19 against 22.5 us: more, shorter work items on an
// otherwise idle device), beyond that the wide ones (41 blocks: 25 against 31 us; 143: 63 against 76), which stage a
// block's rows once per 128 channels.  The count picks, by the number of wide work items.
template <int DT, bool FUSED, bool ADD, int NBW>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void conv3_mixed_kernel(ConvParams p, Plan3 qw, Plan3 qn) {
    const int nact = max(min(*p.count, p.cap), 0);
    if ((uint32_t)nact * (uint32_t)(qw.mpasses * qw.ngroups) >= (uint32_t)p.wide_min_items) {
        // (128 pixels x 128 channels: a wave takes 64 x 64, four fragment reads per four MFMAs, rather than 32 x 128, five)
        if (NBW == 4) conv3_body<DT, FUSED, ADD, 16, 2, 2, 2, 5, 3, true>(p, qw);
        else conv3_body<DT, FUSED, ADD, 16, 4, NBW, 1, 5, 3, true>(p, qw);
    } else {
        conv3_body<DT, FUSED, ADD, 16, 4, 2, 1, 5, 3, true>(p, qn);
    }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
struct Shape3 {
    int pp;          // output pixels per pass
    int cc;          // input channels per chunk
    int nvi;         // input vectors per thread and chunk the kernel is built for
    int nb;          // 32-channel blocks per output group: 2, or 3 / 4 (wide groups)
    bool ok;
    Plan3 q;
    size_t lds_bytes;
};

static Shape3 plan3(const ConvParams &p, int pp, int nb = 2, bool only16 = false) {
    Shape3 sh;
    sh.pp = pp;
    sh.nb = nb;
    sh.ok = false;
    Plan3 &q = sh.q;
    const long long M = (long long)p.oh * p.ow;
    const int CinP = (p.Cin + 31) / 32 * 32;
    q.mpasses = (int)((M + pp - 1) / pp);
    const int gw = nb * 32;
    q.ngroups = (p.Cout + gw - 1) / gw;
    q.div_pt = make_fastdiv((uint32_t)q.mpasses * q.ngroups);
    q.div_ng = make_fastdiv((uint32_t)q.ngroups);
    q.div_sw = make_fastdiv((uint32_t)p.sw);
    // input rows a pass of pp consecutive output pixels can touch
    long long out_rows = (pp + p.ow - 1) / p.ow + ((pp % p.ow) ? 1 : 0);
    if (out_rows > p.oh) out_rows = p.oh;
    long long rows = (out_rows - 1) * p.sh + p.kh;
    if (rows > p.th) rows = p.th;
    q.cpp = (p.tw + p.sw - 1) / p.sw;
    const int taps = p.kh * p.kw;
    q.ks16 = taps * (CinP / 16);
    q.w_bytes = (uint32_t)((size_t)((p.Cout + 63) / 64) * q.ks16 * 2048);      // the packed weights: groups of 64 channels
    const size_t bias_bytes = (size_t)q.ngroups * gw * 4;
    // chunks of 32 channels with up to 6 input vectors per thread, else of 16 with up to 9 (kernels are built for
    // 3 / 6 and 5 / 9: every vector costs its staging instructions whether it carries data or not); two buffers must fit
    // a pointwise kernel has one tap: chunks of 64 channels (up to 9 vectors per thread; kernels built for 5 / 9) keep
    // four MFMA steps in a chunk; channel counts that are no multiple of 64 take chunks of 32
    for (int cc = (taps == 1 ? 64 : 32); cc >= (taps == 1 ? 32 : 16); cc -= (taps == 1 ? 32 : 16)) {
        if (CinP % cc) continue;
        if ((nb > 2 || only16) && cc != 16) continue;  // wide groups (and what runs beside them): built for 16-channel chunks of up to 5 vectors
        const long long nvec = rows * p.tw * (cc / 8);
        const long long need = (nvec + 255) / 256;
        if (pp == 384) {                              // built for 7 vectors of 32 channels or 5 of 16
            if (need > (cc == 32 ? 7 : 5)) continue;
            sh.nvi = cc == 32 ? 7 : 5;
        } else if (nb > 2 || only16) {
            if (need > 5) continue;
            sh.nvi = 5;
        } else {
            if (need > (cc == 32 ? 6 : 9)) continue;
            sh.nvi = cc == 32 ? (need <= 3 ? 3 : 6) : (need <= 5 ? 5 : 9);
        }
        const long long in_b = rows * p.sw * q.cpp * (cc * 2 + 16);
        const long long buf = in_b + (long long)taps * (cc / 16) * nb * 1024;
        const long long total = 2 * buf + kDump3 + 4 * kOst3 + (long long)bias_bytes;
        if (total > kLds3) continue;
        sh.cc = cc;
        q.nvec_in = (uint32_t)nvec;
        q.nchunks = CinP / cc;
        q.div_nch = make_fastdiv((uint32_t)q.nchunks);
        q.w_off = (uint32_t)in_b;
        q.buf_bytes = (uint32_t)buf;
        q.dump_off = 2u * q.buf_bytes;
        q.ost_off = q.dump_off + kDump3;
        q.bias_off = q.ost_off + 4 * kOst3;
        sh.lds_bytes = (size_t)total;
        sh.ok = true;
        break;
    }
    return sh;
}

template <int DT, bool FUSED, bool ADD, int WP, int CBW, int PBW>
static void launch3_cc(const ConvParams &p, const Shape3 &sh, int grid, hipStream_t s) {
#define SBNET_L3(CC, NVI)                                                                                      \
    do {                                                                                                       \
        auto kern = conv3_kernel<DT, FUSED, ADD, CC, WP, CBW, PBW, NVI>;                                       \
        if (sh.lds_bytes > 48 * 1024)                                                                          \
            (void)hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,          \
                                      (int)sh.lds_bytes);                                                      \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(512), sh.lds_bytes, s, p, sh.q);                             \
    } while (0)
    if (p.kh == 1) {                                  // pointwise
#define SBNET_L1(CC, NVI)                                                                                      \
    do {                                                                                                       \
        auto kern = conv3_pointwise_kernel<DT, FUSED, ADD, CC, WP, CBW, PBW, NVI>;                             \
        if (sh.lds_bytes > 48 * 1024)                                                                          \
            (void)hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,          \
                                      (int)sh.lds_bytes);                                                      \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(256), sh.lds_bytes, s, p, sh.q);                             \
    } while (0)
        if (sh.cc == 64 && sh.nvi == 5) SBNET_L1(64, 5);
        else if (sh.cc == 64) SBNET_L1(64, 9);
        else if (sh.nvi == 3) SBNET_L1(32, 3);
        else SBNET_L1(32, 6);
#undef SBNET_L1
    } else if (sh.cc == 32 && sh.nvi == 3) SBNET_L3(32, 3);
    else if (sh.cc == 32) SBNET_L3(32, 6);
    else if (sh.nvi == 5) SBNET_L3(16, 5);
    else SBNET_L3(16, 9);
#undef SBNET_L3
}

template <int DT, bool FUSED, bool ADD>
static void launch3_shape(const ConvParams &p, const Shape3 &sh, int grid, hipStream_t s) {
    if (sh.pp == 256) launch3_cc<DT, FUSED, ADD, 4, 2, 2>(p, sh, grid, s);
    else if (sh.pp == 128) launch3_cc<DT, FUSED, ADD, 4, 2, 1>(p, sh, grid, s);
    else launch3_cc<DT, FUSED, ADD, 2, 1, 1>(p, sh, grid, s);
}

static void launch3(sbnet_dtype dt, bool fused, const ConvParams &p, const Shape3 &sh, hipStream_t s) {
    long long items = (long long)p.cap * sh.q.mpasses * sh.q.ngroups;
    long long g = (items + 7) / 8 * 8;
    const long long most = p.kh == 1 && 2 * sh.lds_bytes <= (size_t)kLds3 ? 512 : 256;   // persistent workgroups: one per CU, two for pointwise
    if (g > most) g = most;
    const int grid = (int)g;
    if (dt == SBNET_BF16) {
        if (fused && p.add) launch3_shape<SBNET_BF16, true, true>(p, sh, grid, s);
        else if (fused) launch3_shape<SBNET_BF16, true, false>(p, sh, grid, s);
        else launch3_shape<SBNET_BF16, false, false>(p, sh, grid, s);
    } else {
        if (fused && p.add) launch3_shape<SBNET_F16, true, true>(p, sh, grid, s);
        else if (fused) launch3_shape<SBNET_F16, true, false>(p, sh, grid, s);
        else launch3_shape<SBNET_F16, false, false>(p, sh, grid, s);
    }
}

template <int DT, bool FUSED, bool ADD, int CCB, int NVIB, int PBWB = 2, int PBWS = 1>
static void launch3_pair_small(const ConvParams &p, const Shape3 &big, const Shape3 &small, int grid, size_t lds, hipStream_t s) {
#define SBNET_L3P(CCS, NVIS)                                                                                   \
    do {                                                                                                       \
        auto kern = conv3_pair_kernel<DT, FUSED, ADD, CCB, NVIB, CCS, NVIS, PBWB, PBWS>;                       \
        if (lds > 48 * 1024)                                                                                   \
            (void)hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
        ConvParams pt = p;                                                                                     \
        pt.small_cost8 = tuning().conv3_small_item_cost_eighths;                                               \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(512), lds, s, pt, big.q, small.q);                           \
    } while (0)
    if (small.cc == 32 && small.nvi == 3) SBNET_L3P(32, 3);
    else if (small.cc == 32) SBNET_L3P(32, 6);
    else if (small.nvi == 5) SBNET_L3P(16, 5);
    else SBNET_L3P(16, 9);
#undef SBNET_L3P
}

template <int DT, bool FUSED, bool ADD>
static void launch3_pair_big(const ConvParams &p, const Shape3 &big, const Shape3 &small, int grid, size_t lds, hipStream_t s) {
    if (big.pp == 384) {                              // planned only for the fused form without the add
        if constexpr (FUSED && !ADD) {
            if (big.cc == 32) launch3_pair_small<DT, FUSED, ADD, 32, 7, 3, 2>(p, big, small, grid, lds, s);
            else launch3_pair_small<DT, FUSED, ADD, 16, 5, 3, 2>(p, big, small, grid, lds, s);
        }
        return;
    }
    if (big.cc == 32 && big.nvi == 3) launch3_pair_small<DT, FUSED, ADD, 32, 3>(p, big, small, grid, lds, s);
    else if (big.cc == 32) launch3_pair_small<DT, FUSED, ADD, 32, 6>(p, big, small, grid, lds, s);
    else if (big.nvi == 5) launch3_pair_small<DT, FUSED, ADD, 16, 5>(p, big, small, grid, lds, s);
    else launch3_pair_small<DT, FUSED, ADD, 16, 9>(p, big, small, grid, lds, s);
}

// both tile shapes in one launch
static void launch3_pair(sbnet_dtype dt, bool fused, const ConvParams &p, const Shape3 &big, const Shape3 &small, hipStream_t s) {
    const long long items = (long long)p.cap * small.q.mpasses * small.q.ngroups;     // the smaller tile has more items
    long long g = (items + 7) / 8 * 8;
    if (g > 256) g = 256;                             // one persistent workgroup per CU
    const int grid = (int)g;
    const size_t lds = big.lds_bytes > small.lds_bytes ? big.lds_bytes : small.lds_bytes;
    if (dt == SBNET_BF16) {
        if (fused && p.add) launch3_pair_big<SBNET_BF16, true, true>(p, big, small, grid, lds, s);
        else if (fused) launch3_pair_big<SBNET_BF16, true, false>(p, big, small, grid, lds, s);
        else launch3_pair_big<SBNET_BF16, false, false>(p, big, small, grid, lds, s);
    } else {
        if (fused && p.add) launch3_pair_big<SBNET_F16, true, true>(p, big, small, grid, lds, s);
        else if (fused) launch3_pair_big<SBNET_F16, true, false>(p, big, small, grid, lds, s);
        else launch3_pair_big<SBNET_F16, false, false>(p, big, small, grid, lds, s);
    }
}

// groups of 96 / 128 channels: both tile shapes in one launch, or the 128-pixel shape alone where the 256-pixel one does
// not fit LDS (the 33x33 input tile of a strided 16x16 block)
constexpr int kWideMinItems = 96;            // wide groups from this many of their work items (see conv3_mixed_kernel)

template <int DT, bool FUSED, bool ADD, int NBW>
static void launch3_wide_nb(const ConvParams &p, const Shape3 &big, const Shape3 &small, hipStream_t s) {
    const long long items = (long long)p.cap * small.q.mpasses * small.q.ngroups;
    long long g = (items + 7) / 8 * 8;
    if (g > 256) g = 256;
    if (big.ok) {
        const size_t lds = big.lds_bytes > small.lds_bytes ? big.lds_bytes : small.lds_bytes;
        auto kern = conv3_pair_kernel<DT, FUSED, ADD, 16, 5, 16, 5, 2, 1, NBW>;
        if (lds > 48 * 1024) (void)hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        ConvParams pt = p;
        pt.small_cost8 = tuning().conv3_small_item_cost_eighths;
        hipLaunchKernelGGL(kern, dim3((int)g), dim3(512), lds, s, pt, big.q, small.q);
    } else {
        // beside the 128-pixel shape with 64-channel groups (same rows, same chunks: it fits where the wide one does)
        const Shape3 narrow = plan3(p, 128, 2, true);
        const long long n_items = (long long)p.cap * narrow.q.mpasses * narrow.q.ngroups;
        long long gn = (n_items + 7) / 8 * 8;
        if (gn > 256) gn = 256;
        const size_t lds = small.lds_bytes > narrow.lds_bytes ? small.lds_bytes : narrow.lds_bytes;
        auto kern = conv3_mixed_kernel<DT, FUSED, ADD, NBW>;
        if (lds > 48 * 1024) (void)hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        ConvParams pt = p;
        pt.wide_min_items = kWideMinItems;
        hipLaunchKernelGGL(kern, dim3((int)gn), dim3(512), lds, s, pt, small.q, narrow.q);
    }
}

template <int DT>
static void launch3_wide(bool fused, const ConvParams &p, const Shape3 &big, const Shape3 &small, hipStream_t s) {
#define SBNET_L3W(FU, AD)                                                                   \
    do {                                                                                    \
        if (small.nb == 3) launch3_wide_nb<DT, FU, AD, 3>(p, big, small, s);                \
        else launch3_wide_nb<DT, FU, AD, 4>(p, big, small, s);                              \
    } while (0)
    if (fused && p.add) SBNET_L3W(true, true);
    else if (fused) SBNET_L3W(true, false);
    else SBNET_L3W(false, false);
#undef SBNET_L3W
}

bool conv3_try(sbnet_dtype dt, bool fused, const ConvParams &p0, hipStream_t s, sbnet_status *st, const char *who) {
    if (dt != SBNET_BF16 && dt != SBNET_F16) return false;
    if (p0.kh != p0.kw || (p0.kh != 3 && p0.kh != 1)) return false;
    if (p0.Cin % 8 != 0 || p0.Cout % 8 != 0) return false;
    // byte offsets inside one sample (fused) or one tile are kept in 32 bits and checked by the hardware
    // against a buffer descriptor of that size
    if ((fused ? (long long)p0.H * p0.W : (long long)p0.th * p0.tw) * p0.Cin >= (1LL << 30)) return false;
    if ((fused ? (long long)p0.Ho * p0.Wo : (long long)p0.oh * p0.ow) * p0.Cout >= (1LL << 30)) return false;
    ConvParams p = p0;
    p.CinP = (p.Cin + 31) / 32 * 32;
    const long long M = (long long)p.oh * p.ow;
    if ((long long)((p.Cout + 63) / 64) * p.kh * p.kw * (p.CinP / 16) * 2048 >= (1LL << 31)) return false;

    Shape3 big, small;
    big.ok = small.ok = false;
    if (M <= 64) {
        big = plan3(p, 64);
    } else if (p.kh == 1) {
        // pointwise: one shape, chosen on the host; a smaller tile if that lets two workgroups share a CU
        big = plan3(p, M > 128 ? 256 : 128);
        if (!big.ok || 2 * big.lds_bytes > (size_t)kLds3) {
            Shape3 alt = plan3(p, 128);
            if (alt.ok && (!big.ok || 2 * alt.lds_bytes <= (size_t)kLds3)) big = alt;
        }
    } else {
        // Strided tiles of up to 256 pixels whose rows fit in 16-channel chunks of five vectors per thread: groups of 128
        // output channels where the channel count is a multiple of that, of 96 where that spares a half-empty group of
        // 64 (96, 288 ...).  Measured on the stage shapes: stride 1 gains nothing from them (96 -> 96) or loses (192 -> 192:
        // its rows fit 32-channel chunks with 64-channel groups, twice the matrix steps per barrier), 96 -> 192 at
        // stride 2 is the same with either.
        const int nbw = p.Cout % 128 == 0 ? 4 : (p.Cout % 96 == 0 && p.Cout % 64 != 0 ? 3 : 2);
        if (nbw > 2 && M <= 256 && p.sh > 1) {
            Shape3 wb, ws = plan3(p, 128, nbw);
            wb.ok = false;
            if (M > 128) wb = plan3(p, 256, nbw);
            // (without a 256-pixel wide shape the launch also holds the 128-pixel shape with 64-channel groups)
            if (ws.ok && (wb.ok || plan3(p, 128, 2, true).ok) &&
                (long long)p.cap * ws.q.mpasses * ((p.Cout + 63) / 64) < (1LL << 31)) {
                if (wb.ok && (long long)p.cap * ws.q.mpasses * ws.q.ngroups <= 256) wb.ok = false;    // as below
                if (dt == SBNET_BF16) launch3_wide<SBNET_BF16>(fused, p, wb, ws, s);
                else launch3_wide<SBNET_F16>(fused, p, wb, ws, s);
                *st = launch_status(who);
                return true;
            }
        }
        if (M > 256 && M <= 384 && fused && !p.add) {          // 384 pixels beside 256, if the count can ever pick 384
            const Shape3 b3 = plan3(p, 384), s2 = plan3(p, 256);
            if (b3.ok && s2.ok && (long long)p.cap * s2.q.mpasses * s2.q.ngroups > 256) {
                big = b3;
                small = s2;
            }
        }
        if (!big.ok) {                                         // 256 pixels beside 128
            if (M > 128) big = plan3(p, 256);
            small = plan3(p, 128);
        }
    }
    if (!big.ok && !small.ok) return false;
    const int most_passes = small.ok ? small.q.mpasses : big.q.mpasses;          // the smaller tile has more of them
    if ((long long)p.cap * most_passes * ((p.Cout + 63) / 64) >= (1LL << 31)) return false;
    // with at most 256 items of the smaller tile whatever the count, the rule in the kernel never picks the larger one
    if (big.ok && small.ok && (long long)p.cap * small.q.mpasses * small.q.ngroups <= 256) big.ok = false;
    if (big.ok && small.ok) launch3_pair(dt, fused, p, big, small, s);     // the device-side count picks the shape
    else if (big.ok) launch3(dt, fused, p, big, s);
    else launch3(dt, fused, p, small, s);
    *st = launch_status(who);
    return true;
}

}  // namespace sbnet
