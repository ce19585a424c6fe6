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
//   * global memory is reached through buffer descriptors that cover one sample (or one tile):
//     a halo pixel above or below the image lands outside the descriptor, one to the left or
//     right gets an out-of-range offset on purpose, and the hardware returns zeros for such loads
//     and drops such stores.  The tile loop therefore has no branch and no predicate around any
//     memory operation, and the compiler's wait counts stay exact (with branches they turn into
//     full waits and every load or store then costs its own memory round trip);
//   * the 18x18xCIN input sub-tile (block + halo) is double-buffered in LDS and software-pipelined
//     two tiles deep: while the matrix cores work on tile i, the same wave, between its MFMAs,
//     writes tile i+1 (loaded during tile i-1) to the other LDS buffer and issues the loads of
//     tile i+2 into the registers this frees.  The index triple of tile i+3 is requested at the
//     same time.  No load waits on another load.  Per stage of 12 MFMAs this adds one LDS write, one
//     buffer load and five VALU instructions (measured: a wave issues about two VALU instructions
//     per MFMA for free, every further one delays the next MFMA by its own four cycles);
//   * results leave through a wave-private LDS transpose, so that a store instruction writes 64-byte
//     runs instead of 16-byte pieces, and as non-temporal stores;
//   * a workgroup with a single tile (fewer active tiles than CUs) runs a copy of the tile code
//     that starts its matrix work while the weights, requested in order of use, still stream in;
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
constexpr int kOutPs = 80;                       // LDS bytes per pixel of a wave's results: 32 channels + 16 B pad

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

// ADD (fused form only): the results are added to what the output holds.  A template parameter rather than a
// branch on p.add: with two paths that issue different numbers of memory operations the compiler's wait counts
// after the join are those of the shorter path, and the first LDS write of the next tile then waits for this
// tile's stores to be acknowledged.
// FLAGS (fused form, 16 x 16 blocks only): the active blocks come as one flag byte per block instead of an index
// list.  Every wave counts the flags in its prologue (16 per lane and load, prefix sums across the lanes) and
// notes the blocks of its workgroup's items in LDS; the workgroups also write the index triples of their items
// and the count, so that the call leaves behind what reduce_mask would have.  This replaces reduce_mask's second launch, and the count
// and index loads of the plain form, by work that overlaps the arrival of the weights.
constexpr int kMineMax = 256;            // items per workgroup in the flag-fed form: 65 536 blocks / 256 workgroups

template <int DT, int CIN, bool FUSED, bool ADD, bool FLAGS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void conv16_kernel(ConvParams p, Sub16 sp) {
    static_assert(FUSED || !ADD, "adding into the output is part of the fused form");
    static_assert(FUSED || !FLAGS, "flags replace the index list of the fused form");
    constexpr int KC = CIN / 16;                     // 16-channel k-steps per tap
    constexpr int CV = CIN / 8;                      // 16-byte vectors per pixel
    constexpr int PS = (CIN + 8) * 2;                // LDS bytes per pixel
    constexpr int NVEC = kT16Px * CV;
    constexpr int NV = (NVEC + 255) / 256;           // staging vectors per thread
    constexpr int PXK = 256 / CV;                    // pixels between a thread's consecutive vectors
    constexpr int LPX = NV * PXK;                    // pixels per LDS buffer: every staging vector has a slot
    constexpr int KS = 9 * KC;
    constexpr int NST = 3 * KC;                      // pipeline stages: (tap column, channel step)
    static_assert(NV <= NST, "one staging vector per pipeline stage");
    __shared__ __align__(16) unsigned char lds[2][LPX * PS];
    __shared__ __align__(16) unsigned char ostage[4][8 * 16 * kOutPs];       // per wave: 8 rows x 16 pixels of results
    __shared__ uint32_t mine_all[4][FLAGS ? kMineMax : 1];      // FLAGS: block number of this workgroup's k-th item, one copy per wave

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 5, m = lane & 31;          // k-group / channel group, pixel within a fragment
    const int prow = m >> 4, pcol = m & 15;
    const int rh = wave >> 1, nh = wave & 1;
    const int ng = blockIdx.y;
    uint32_t *mine = mine_all[wave];
    const uint32_t per_block = (uint32_t)sp.sub_h * sp.sub_w;
    const uint32_t G = gridDim.x;                    // multiple of 8
    // workgroups are dealt round-robin to the 8 XCDs: give each XCD a contiguous run of items
    const uint32_t first = (blockIdx.x & 7) * (G >> 3) + (blockIdx.x >> 3);

    // A work item's index triple is requested well before it is needed.  The address is the same in
    // every lane, but the loads are issued as per-lane loads and left in vector registers (the opaque
    // zero hides the uniformity): a value the compiler knows to be uniform is moved to a scalar
    // register right after the load, which would stall the wave for the memory round trip on the spot.
    int lane_zero = 0;
    asm volatile("" : "+v"(lane_zero));
    auto request = [&](uint32_t it) __attribute__((always_inline)) {
        Item16 c;
        c.b = fdiv(it, sp.div_sub);
        const uint32_t sidx = it - c.b * per_block;
        c.si = (int)fdiv(sidx, sp.div_subw);
        c.sj = (int)sidx - c.si * sp.sub_w;
        c.n = c.by = c.bx = 0;
        if (FLAGS) {
            const uint32_t k = fdiv(it - first, p.div_grid);         // this workgroup's k-th item
            const uint32_t blk = mine[k + lane_zero];
            c.n = (int)fdiv(blk, p.div_bps);
            const uint32_t rem = blk - (uint32_t)c.n * (uint32_t)(p.g_in.bcount_h * p.g_in.bcount_w);
            c.by = (int)fdiv(rem, p.div_bw);
            c.bx = (int)rem - c.by * p.g_in.bcount_w;
        } else if (FUSED) {
            const int32_t *t = p.indices + 3 * (size_t)c.b + lane_zero;
            c.n = t[0];
            c.by = t[1];
            c.bx = t[2];
        }
        return c;
    };
    auto resolve = [&](const Item16 &c) __attribute__((always_inline)) {
        Item16 r = c;
        if (FUSED) {
            r.n = __builtin_amdgcn_readfirstlane(c.n);
            r.by = __builtin_amdgcn_readfirstlane(c.by);
            r.bx = __builtin_amdgcn_readfirstlane(c.bx);
        }
        return r;
    };

    // ---- Prologue.  Order of the requests (loads return in the order they were issued, and a workgroup's four
    //      waves share one address unit that takes 16 cycles per 16-byte load instruction, so a wave's 36 weight
    //      loads alone keep it busy for ~2300 cycles):
    //        1. the few bytes the block list hangs on (count and first index triple, or the flags),
    //        2. the bias and the weights of the first stages,
    //        3. (after the list is known) the first tile,
    //        4. the weights of the next few stages; the rest follows once the tile is in LDS (a workgroup with a
    //           single tile requests them between its first MFMAs): they stream in faster than the matrix work
    //           consumes them, and a wave that is busy issuing loads cannot move its tile to LDS.
    //      Everything that does not depend on the block list is computed while those first bytes are on their way.
    int nact_raw = 0;
    constexpr int kEarly = 4;                         // flag vectors per lane requested up front: 4096 blocks
    uint4 fl[kEarly];                                 // indexed by constants only: stays in registers
    Item16 cur;
    if (FLAGS) {
        // no branch around a load (the wave would wait for it on the spot): the vector number is clamped into the
        // flag buffer and what lies behind the last block is dropped when the flags are counted
        const int last_vec = (p.total_blocks - 1) >> 4;
#pragma unroll
        for (int r = 0; r < kEarly; ++r) fl[r] = reinterpret_cast<const uint4 *>(p.flags)[min(lane * kEarly + r, last_vec)];
    } else {
        // The count and the first index triple are independent loads (the index is clamped into the
        // buffer), so their latencies overlap instead of chaining.  Items past the end repeat the last
        // one: its loads are harmless and nothing is stored for it (the loop has ended by then).
        nact_raw = *p.count;
        cur = request(min(first, (uint32_t)p.cap * per_block - 1u));
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
    // weights of this wave: every k-step of its 32 output channels
    uint4 wreg[KS];
    const uint4 *wsrc = (const uint4 *)p.w + p.w32_offset + ((size_t)ng * KS * 2 + nh) * 64 + lane;
    auto wload1 = [&](int st, int r) __attribute__((always_inline)) {       // k-step of tap row r that stage st multiplies with
        const int ks = (r * 3 + st / KC) * KC + st % KC;
        wreg[ks] = wsrc[(size_t)ks * 128];
    };
    auto wload = [&](int st) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < 3; ++r) wload1(st, r);
    };
    constexpr int kWFirst = 1;                        // stages whose weights go ahead of the first tile,
    constexpr int kWPro = NST < 3 ? NST : 3;          // ... and stages whose weights are requested before its matrix work starts
#pragma unroll
    for (int st = 0; st < kWFirst; ++st) wload(st);
    __builtin_amdgcn_sched_barrier(0);

    // ---- staging plan, the same for every tile: vector k of this thread is 16 bytes of pixel px0 + k*PXK
    //      of the 18x18 sub-tile (LDS has slots for the few pixel numbers past the end).
    const int in_w = FUSED ? p.W : p.tw;                         // pixels per row of the addressed array
    const uint32_t in_bytes = (uint32_t)(FUSED ? p.H : p.th) * in_w * CIN * 2u;      // one sample / one tile
    uint32_t delta[NV];                                          // byte offset from the sub-tile origin
    int colk[NV];                                                // column inside the sub-tile
    {
        const int px0 = threadIdx.x / CV, c8 = threadIdx.x % CV;
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const int px = px0 + k * PXK;
            const int row = px / kT16, col = px % kT16;
            delta[k] = (uint32_t)((row * in_w + col) * CIN + c8 * 8) * 2u;
            colk[k] = col;
        }
    }
    struct Src {
        __amdgpu_buffer_rsrc_t rsrc;     // the sample (fused) or tile that holds the sub-tile
        uint32_t origin;                 // byte offset of the sub-tile's pixel (0, 0); wraps below zero above / left of the image
        int gx0;                         // image column of sub-tile column 0
    };
    auto source = [&](const Item16 &c) __attribute__((always_inline)) {
        Src s;
        const uint16_t *base = (const uint16_t *)p.in;
        int y0, x0;
        if (FUSED) {
            y0 = p.g_in.boffset_h + c.by * p.g_in.bstride_h + c.si * 16;
            x0 = p.g_in.boffset_w + c.bx * p.g_in.bstride_w + c.sj * 16;
            base += (long long)c.n * p.H * p.W * CIN;
        } else {
            y0 = c.si * 16;
            x0 = c.sj * 16;
            base += (long long)c.b * p.th * p.tw * CIN;
        }
        s.rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, (int)in_bytes, (int)kBufWord3);
        s.origin = (uint32_t)((y0 * in_w + x0) * CIN) * 2u;
        s.gx0 = x0;
        return s;
    };
    // Rows outside the image fall outside the descriptor by themselves; columns outside would wrap
    // into the neighbouring row, so they get the out-of-range offset.  Either way the load returns zeros.
    uint4 stage[NV];
    auto fetch1 = [&](const Src &s, int k) __attribute__((always_inline)) {
        const bool col_ok = !FUSED || (uint32_t)(s.gx0 + colk[k]) < (uint32_t)p.W;
        stage[k] = buf_load16(s.rsrc, col_ok ? s.origin + delta[k] : kOutOfRange);
    };
    const uint32_t stash_off = (threadIdx.x / CV) * PS + (threadIdx.x % CV) * 16;
    auto stash1 = [&](int buf, int k) __attribute__((always_inline)) {
        *(uint4 *)(&lds[buf][stash_off + k * PXK * PS]) = stage[k];
    };
    __builtin_amdgcn_sched_barrier(0);

    uint32_t kk = 0;                                 // FLAGS: number of this workgroup's items
    if (FLAGS) {
        // Compaction of the flag bytes (each 0 or 1, the padding behind the last block 0).  Every wave does all of it
        // for itself, 4096 blocks per round: a lane takes 64 consecutive flags, a prefix sum over the lanes and the
        // rounds gives the list positions [excl, excl + c) of its active blocks.  This workgroup's items are the
        // positions first, first + G, ...; G is at least 64, so a lane's run holds at most one of them, and every lane
        // looks for its own in parallel: k = ceil((excl - first) / G), and if first + k G lies in the run, the block is
        // the (first + k G - excl)-th set flag of the lane's 64, found by halving.  The table the blocks go to is the
        // wave's own: no barrier and no exchange between waves, some sixty instructions per round whatever the number
        // of items.  per_block is 1 in this form: list position = item number.
        int running = 0;
        static_assert(kEarly == 4, "the scan takes four flag vectors per lane and round");
        auto count16 = [](uint4 v) __attribute__((always_inline)) { return __popc(v.x) + __popc(v.y) + __popc(v.z) + __popc(v.w); };
        // (the four vectors travel as values, not as an array: an array indexed at run time would live in scratch memory)
        auto scan_round = [&](uint4 q0, uint4 q1, uint4 q2, uint4 q3, int b0) __attribute__((always_inline)) {
            const int c0 = b0 < p.total_blocks ? count16(q0) : 0, c1 = b0 + 16 < p.total_blocks ? count16(q1) : 0;
            const int c2 = b0 + 32 < p.total_blocks ? count16(q2) : 0, c3 = b0 + 48 < p.total_blocks ? count16(q3) : 0;
            const int c = c0 + c1 + c2 + c3;
            const int incl = wave_inclusive_sum(c);
            const int excl = running + incl - c;
            const uint32_t k = excl > (int)first ? fdiv((uint32_t)excl - first + G - 1u, p.div_grid) : 0u;
            const int pos = (int)(first + k * G);                        // the first own position not in front of the run
            if (pos < excl + c && pos < p.cap) {                         // (pos >= excl by construction)
                int skip = pos - excl, at = 0;
                uint4 v = q0;
                if (skip >= c0) { skip -= c0; v = q1; at = 16;
                    if (skip >= c1) { skip -= c1; v = q2; at = 32;
                        if (skip >= c2) { skip -= c2; v = q3; at = 48; } } }
                // the 0/1 bytes of a word gathered into four neighbouring bits by one multiplication
                uint32_t bits = ((v.x * 0x01020408u) >> 24) | (((v.y * 0x01020408u) >> 24) << 4) |
                                (((v.z * 0x01020408u) >> 24) << 8) | (((v.w * 0x01020408u) >> 24) << 12);
#pragma unroll
                for (int half = 8; half >= 1; half >>= 1) {              // the skip-th set bit, by halving
                    const int below = __popc(bits & ((1u << half) - 1u));
                    if (skip >= below) { skip -= below; bits >>= half; at += half; }
                }
                mine[k] = (uint32_t)(b0 + at);                           // k < kMineMax: checked on the host
            }
            running += __builtin_amdgcn_readlane(incl, 63);
        };
        scan_round(fl[0], fl[1], fl[2], fl[3], lane * kEarly * 16);
        for (int c0 = kEarly * 1024; c0 < p.total_blocks; c0 += kEarly * 1024) {
            const int b0 = c0 + lane * kEarly * 16;
            const int last_vec = (p.total_blocks - 1) >> 4;
            const uint4 *fv = reinterpret_cast<const uint4 *>(p.flags);
            const uint4 q0 = fv[min((b0 >> 4) + 0, last_vec)], q1 = fv[min((b0 >> 4) + 1, last_vec)];
            const uint4 q2 = fv[min((b0 >> 4) + 2, last_vec)], q3 = fv[min((b0 >> 4) + 3, last_vec)];
            scan_round(q0, q1, q2, q3, b0);
        }
        nact_raw = running;
    }
    const uint32_t items = (uint32_t)max(min(nact_raw, p.cap), 0) * per_block;
    if (FLAGS && first < items) kk = fdiv(items - 1u - first, p.div_grid) + 1u;
    if (first >= items) {
        // no item: all that is left is the count, should this be the workgroup that reports it
        if (FLAGS && blockIdx.x == 0 && ng == 0 && threadIdx.x == 0) *p.count_out = nact_raw;
        return;
    }
    const uint32_t last = items - 1u;
    if (FLAGS) cur = request(first);
    Item16 nx1 = request(min(first + G, last));
    Item16 nx2 = request(min(first + 2 * G, last));
    cur = resolve(cur);

    Src src = source(cur);
#pragma unroll
    for (int k = 0; k < NV; ++k) fetch1(src, k);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int st = kWFirst; st < kWPro; ++st) wload(st);
    __builtin_amdgcn_sched_barrier(0);

    if (FLAGS && ng == 0 && wave == 0) {
        // what reduce_mask would have left behind: every workgroup writes the index triples of its own items
        // (together they are the whole list up to cap), one lane the count
        for (uint32_t k = lane; k < kk; k += 64) {
            const uint32_t blk = mine[k];
            const int n = (int)fdiv(blk, p.div_bps);
            const uint32_t rem = blk - (uint32_t)n * (uint32_t)(p.g_in.bcount_h * p.g_in.bcount_w);
            const int by = (int)fdiv(rem, p.div_bw);
            int32_t *t = p.indices_out + 3 * ((size_t)first + (size_t)k * G);
            t[0] = n;
            t[1] = by;
            t[2] = (int)rem - by * p.g_in.bcount_w;
        }
        if (blockIdx.x == 0 && lane == 0) *p.count_out = nact_raw;
    }

    // ReLU as an integer max on the float bits (negative floats are negative integers); without
    // ReLU the floor is INT_MIN and the max is the identity.  One VALU op, no NaN canonicalisation.
    int floor_i = p.relu ? 0 : (int)0x80000000;
    asm volatile("" : "+s"(floor_i));                // opaque: otherwise the max is split into a max with 0 and a select
    uint32_t floor16 = p.relu ? 0u : 0x80008000u;    // the same for two 16-bit values at once
    asm volatile("" : "+s"(floor16));

    // ---- output plan: this lane stores pixel (rh*8 + 2P + prow, pcol) of the sub-tile, channels ch0 .. ch0+15
    const int out_w = FUSED ? p.Wo : p.ow;
    const uint32_t out_bytes = (uint32_t)(FUSED ? p.Ho : p.oh) * out_w * p.Cout * 2u;
    const uint32_t out_lane = (uint32_t)(((rh * 8 + prow) * out_w + pcol) * p.Cout + ch0) * 2u;
    const uint32_t out_pair = (uint32_t)(2 * out_w * p.Cout) * 2u;          // two rows down
    const bool chan_ok[2] = {ch0 < p.Cout, ch0 + 8 < p.Cout};
    // ... and after the transpose through LDS: pixel (rh*8 + j, lane / 4), 16 bytes number lane % 4 of the
    // wave's 32 channels
    const uint32_t out_row = (uint32_t)(out_w * p.Cout) * 2u;
    const uint32_t out_lane2 = (uint32_t)((rh * 8 * out_w + (lane >> 2)) * p.Cout + ng * 64 + nh * 32 + (lane & 3) * 8) * 2u;
    const bool chan_ok2 = ng * 64 + nh * 32 + (lane & 3) * 8 < p.Cout;
    const uint32_t ost_w = (prow * 16 + pcol) * kOutPs + g * 32;           // MFMA layout -> LDS (+ row pair, half)
    const uint32_t ost_r = (lane >> 2) * kOutPs + (lane & 3) * 16;          // LDS -> store layout (+ row)

    nx1 = resolve(nx1);
#pragma unroll
    for (int k = 0; k < NV; ++k) stash1(0, k);

    // One tile.  A workgroup that has a single tile (the usual case below one tile per CU) runs a copy of this
    // code of its own (SINGLE) that does no staging work for following tiles and is entered while the weights are
    // still on their way: loads return in order and they were requested in the order of use, so the matrix work
    // of a stage waits only for its own weights and overlaps the arrival of the rest.
    int buf = 0;
    auto tile = [&](uint32_t it, auto single_tag) __attribute__((always_inline)) {
        constexpr bool SINGLE = decltype(single_tag)::value;
        Item16 nx3 = nx2;
        if (!SINGLE) {
            nx3 = request(min(it + 3 * G, last));                // used two iterations from now
            nx2 = resolve(nx2);
            src = source(nx2);
        }

        // ---- 16x16 outputs x 64 channels; this wave: 4 output row pairs x 32 channels.
        // Fragment j of a stage holds input rows rh*8 + j, rh*8 + j + 1 (j = 0..8) at tap column t;
        // output row pair P with tap row r reads fragment 2P + r.  Stages are software-pipelined:
        // while the matrix cores consume the nine fragments of one stage, the nine of the next are
        // read from LDS into the other register set.  Between the last MFMAs of stage k the wave also
        // moves staging vector k of the next tile to LDS and reloads it with the tile after that.
        // The scheduling barriers keep all of this interleaved as written.
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
                if (!SINGLE) {
                    if (mm == 9 && st < NV) stash1(buf ^ 1, st);
                    if (mm == 10 && st < NV) fetch1(src, st);
                } else if (mm >= 8 && mm <= 10 && st + kWPro < NST) {
                    wload1(st + kWPro, mm - 8);      // the weights of the later stages arrive while the first ones are used
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }

        // ---- epilogue: ReLU, optional add, NHWC stores.  In the MFMA result layout a lane holds 16 channels of
        //      one pixel and neighbouring lanes hold neighbouring pixels, so storing from it would scatter 16-byte
        //      pieces over 32 cache lines per instruction.  The wave instead transposes its 8 rows x 16 pixels x
        //      32 channels through a private LDS area: afterwards four neighbouring lanes hold the 64 contiguous
        //      bytes of one pixel and a store instruction covers one output row of the wave.
        //      Rows outside the image are outside the descriptor; columns outside and channels past Cout get the
        //      out-of-range offset; the hardware drops those stores (and returns zeros for those loads).
        {
            uint16_t *obase = (uint16_t *)p.out;
            int y0, x0;
            if (FUSED) {
                y0 = p.g_out.boffset_h + cur.by * p.g_out.bstride_h + cur.si * 16;
                x0 = p.g_out.boffset_w + cur.bx * p.g_out.bstride_w + cur.sj * 16;
                obase += (long long)cur.n * p.Ho * p.Wo * p.Cout;
            } else {
                y0 = cur.si * 16;
                x0 = cur.sj * 16;
                obase += (long long)cur.b * p.oh * p.ow * p.Cout;
            }
            const __amdgpu_buffer_rsrc_t orsrc = __builtin_amdgcn_make_buffer_rsrc((void *)obase, 0, (int)out_bytes, (int)kBufWord3);
            const uint32_t origin = (uint32_t)((y0 * out_w + x0) * p.Cout) * 2u;
            uint4 old[4][2];
            if (ADD) {       // read in the MFMA layout, so that the sum is formed in fp32 and rounded once
                const bool col_ok = (uint32_t)(x0 + pcol) < (uint32_t)p.Wo;
#pragma unroll
                for (int P = 0; P < 4; ++P)
#pragma unroll
                    for (int h = 0; h < 2; ++h)
                        old[P][h] = buf_load16(orsrc, (col_ok && chan_ok[h]) ? origin + out_lane + P * out_pair + h * 16 : kOutOfRange);
            }
            unsigned char *os = ostage[wave];
            const bool ok2 = chan_ok2 && (!FUSED || (uint32_t)(x0 + (lane >> 2)) < (uint32_t)p.Wo);
            const uint32_t off2 = ok2 ? origin + out_lane2 : kOutOfRange;
            // Row pair P goes to LDS while the two rows of pair P - 1 come back in the store layout and leave: the
            // LDS round trip of one pair hides behind the conversion of the next.  LDS serves one wave's accesses
            // in order, so a read sees the writes before it without a wait.
#pragma unroll
            for (int P = 0; P <= 4; ++P) {
                if (P < 4) {
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        uint32_t w[4];
                        if (ADD) {
                            float v[8];
#pragma unroll
                            for (int k = 0; k < 8; ++k) v[k] = __int_as_float(max(__float_as_int(acc[P][h * 8 + k]), floor_i));
                            const uint4 o = old[P][h];
                            v[0] += unpack_lo<DT>(o.x); v[1] += unpack_hi<DT>(o.x);
                            v[2] += unpack_lo<DT>(o.y); v[3] += unpack_hi<DT>(o.y);
                            v[4] += unpack_lo<DT>(o.z); v[5] += unpack_hi<DT>(o.z);
                            v[6] += unpack_lo<DT>(o.w); v[7] += unpack_hi<DT>(o.w);
#pragma unroll
                            for (int k = 0; k < 4; ++k) w[k] = pack2<DT>(v[2 * k], v[2 * k + 1]);
                        } else {
                            // ReLU after rounding, two channels per instruction: bf16 and f16 are sign-magnitude, so a
                            // negative value is a negative 16-bit integer and max(., 0) is the ReLU (floor -32768: identity)
#pragma unroll
                            for (int k = 0; k < 4; ++k)
                                w[k] = relu_pair(pack2<DT>(acc[P][h * 8 + 2 * k], acc[P][h * 8 + 2 * k + 1]), floor16);
                        }
                        *(uint4 *)(os + ost_w + P * (2 * 16 * kOutPs) + h * 16) = make_uint4(w[0], w[1], w[2], w[3]);
                    }
                }
                if (P >= 1) {
                    __builtin_amdgcn_wave_barrier();     // no wait: only keeps the compiler from moving reads over writes
#pragma unroll
                    for (int j = 2 * (P - 1); j < 2 * P; ++j) {
                        const uint4 v = *(const uint4 *)(os + ost_r + j * (16 * kOutPs));
                        buf_store16(orsrc, ok2 ? off2 + j * out_row : kOutOfRange, v);
                    }
                }
            }
        }

        if (!SINGLE) {
            __syncthreads();
            buf ^= 1;
            cur = nx1;
            nx1 = nx2;
            nx2 = nx3;
        }
    };
    if (first + G >= items) {                    // workgroup-uniform
        __syncthreads();
        tile(first, std::true_type{});
        return;
    }
#pragma unroll
    for (int st = kWPro; st < NST; ++st) wload(st);
    src = source(nx1);
#pragma unroll
    for (int k = 0; k < NV; ++k) fetch1(src, k);     // tile 1 rides through tile 0's matrix work
    // Every load of the prologue but those has landed before the loop is entered: the loop's wait counts then do
    // not have to allow for prologue loads still in flight.
    __builtin_amdgcn_s_waitcnt(0x0F70 | (NV & 15) | ((NV >> 4) << 14));      // vmcnt(NV)
    __syncthreads();
    for (uint32_t it = first; it < items; it += G) tile(it, std::false_type{});
}

template <int DT, int CIN>
static void launch16(bool fused, const ConvParams &p, const Sub16 &sp, dim3 grid, hipStream_t s) {
    if (fused && p.flags && p.add) hipLaunchKernelGGL((conv16_kernel<DT, CIN, true, true, true>), grid, dim3(256), 0, s, p, sp);
    else if (fused && p.flags) hipLaunchKernelGGL((conv16_kernel<DT, CIN, true, false, true>), grid, dim3(256), 0, s, p, sp);
    else if (fused && p.add) hipLaunchKernelGGL((conv16_kernel<DT, CIN, true, true, false>), grid, dim3(256), 0, s, p, sp);
    else if (fused) hipLaunchKernelGGL((conv16_kernel<DT, CIN, true, false, false>), grid, dim3(256), 0, s, p, sp);
    else hipLaunchKernelGGL((conv16_kernel<DT, CIN, false, false, false>), grid, dim3(256), 0, s, p, sp);
}

// Shape checks and launch shape; false when the shape (or, with p.flags set, the flag-fed form) is not this kernel's.
static bool conv16_plan(sbnet_dtype dt, bool fused, const ConvParams &p, Sub16 *spo, dim3 *grido) {
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
    // byte offsets inside one sample (fused) or one tile are kept in 32 bits and checked by the hardware
    // against a buffer descriptor of that size
    if ((fused ? (long long)p.H * p.W : (long long)p.th * p.tw) * p.Cin >= (1LL << 30)) return false;
    if ((fused ? (long long)p.Ho * p.Wo : (long long)p.oh * p.ow) * p.Cout >= (1LL << 30)) return false;
    long long g = (items + 7) / 8 * 8;
    if (g > 256) g = 256;                             // one persistent workgroup per CU
    if (p.flags) {
        // flag-fed form: list position = item number, a workgroup's items fit its table, block numbers fit the scan
        if (!fused || sp.sub_h != 1 || sp.sub_w != 1 || p.total_blocks > 65536 || p.total_blocks <= 0) return false;
        if (g < 64 || (items + g - 1) / g > kMineMax) return false;      // a lane's 64 flags hold at most one of a workgroup's items
        if (!p.indices_out || !p.count_out) return false;
    }
    *spo = sp;
    *grido = dim3((unsigned)g, (unsigned)((p.Cout + 63) / 64));
    return true;
}

bool conv16_accepts(sbnet_dtype dt, bool fused, const ConvParams &p) {
    Sub16 sp;
    dim3 grid;
    return p.cap > 0 && conv16_plan(dt, fused, p, &sp, &grid);
}

bool conv16_try(sbnet_dtype dt, bool fused, const ConvParams &p, hipStream_t s, sbnet_status *st, const char *who) {
    Sub16 sp;
    dim3 grid;
    if (!conv16_plan(dt, fused, p, &sp, &grid)) return false;
    ConvParams pf = p;
    if (p.flags) {
        pf.div_grid = make_fastdiv(grid.x);
        pf.div_bps = make_fastdiv((uint32_t)p.g_in.bcount_h * (uint32_t)p.g_in.bcount_w);
        pf.div_bw = make_fastdiv((uint32_t)p.g_in.bcount_w);
    }
    if (dt == SBNET_BF16) {
        if (p.Cin == 64) launch16<SBNET_BF16, 64>(fused, pf, sp, grid, s);
        else launch16<SBNET_BF16, 32>(fused, pf, sp, grid, s);
    } else {
        if (p.Cin == 64) launch16<SBNET_F16, 64>(fused, pf, sp, grid, s);
        else launch16<SBNET_F16, 32>(fused, pf, sp, grid, s);
    }
    *st = launch_status(who);
    return true;
}

}  // namespace sbnet
